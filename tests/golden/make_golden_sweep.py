#!/usr/bin/env python3
"""Writes tests/golden/sweep_<config>.json: the CPU oracle's ACDC pass restricted
to a few receivers of one named config (full size), with its evaluation trace.

Only oracle/ and synth/ are used.  The GPU test runs pahq_acdc_sweep on the
same receivers with the same threshold and compares the trace step by step.

usage: python tests/golden/make_golden_sweep.py cfg2 5e-4
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                   # noqa: E402
from oracle.model import Model                 # noqa: E402
from oracle.acdc import Acdc                   # noqa: E402


def receivers_for(name, g, L):
    top = L - 1
    if name == "cfg2":
        return [g.OUT, g.mlpin(top), g.headin(top, 7, 2), g.headin(top, 7, 1), g.headin(top, 2, 0), g.headin(top - 1, 4, 2)]
    raise SystemExit("no receiver sample defined for " + name)


def main():
    name, tau = sys.argv[1], float(sys.argv[2])
    t0 = time.time()
    shape, w, clean, corrupt, spec = synth.make_workload(name)
    oa = Acdc(Model(shape, w), clean, corrupt)
    recv = receivers_for(name, oa.g, shape.n_layers)
    removed, trace = oa.sweep(tau, receivers=recv,
                              progress=lambda v, n, r: print("receiver", v, "evals", n, "removed", r,
                                                             "t=%.0fs" % (time.time() - t0), flush=True))
    out = {"config": name, "seed": spec["seed"], "tau": tau, "receivers": [int(r) for r in recv],
           "trace": [[int(v), int(u), kn, kc, bool(rm)] for v, u, kn, kc, rm in trace],
           "removed": [int(x) for x in oa.g.removed_to_flat(removed).nonzero()[0]]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sweep_%s.json" % name)
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, "evals", len(trace), "removed", len(out["removed"]), "in %.0f s" % (time.time() - t0))


if __name__ == "__main__":
    main()
