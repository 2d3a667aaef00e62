"""Host logic of the sweep under the address and undefined-behaviour sanitizers, on the CPU.

tests/host/controller_check.cpp includes the library's own csrc/controller.h and csrc/graph.h (they hold
no GPU type) and plays the device with a synthetic metric: the accept scan over speculative batches must
reach, decision by decision, what the sequential procedure reaches (paper, Appendix "Preliminaries":
pruning rule), the receiver plans must describe the removed set exactly with the cheaper form, liveness
and the order of receivers must follow their definitions, and an evaluator error must come back.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_controller_under_sanitizers(tmp_path):
    exe = str(tmp_path / "controller_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-I" + os.path.join(ROOT, "paper_2510_23264_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host", "controller_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "0 failures" in r.stdout
