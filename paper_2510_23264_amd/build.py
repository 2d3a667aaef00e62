"""Builds libpahq.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpahq.so")
SOURCES = ["rows.hip", "gemm.hip", "oproj.hip", "attn_kl.hip", "engine.hip", "api.hip", "ceilings.hip", "noalloc.hip"]
# -ffp-contract=off: a product and a sum are rounded separately unless the source says fmaf.  The same
# expression (a norm's x * rstd * gain + offset, a GEMM epilogue's acc * scale + bias) is compiled into
# several kernels -- cache passes and candidate passes take different ones -- and results that must agree
# bit for bit between them (a clean patch scores exactly 0) may not depend on where the compiler chose to fuse.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return obj


def build(verbose=False):
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
