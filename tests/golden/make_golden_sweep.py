#!/usr/bin/env python3
"""Writes tests/golden/sweep_<name>.json: the CPU oracle's literal one-by-one ACDC pass on one named
config (full size), whole or restricted to a few receivers, with its evaluation trace and the removed set
it ends with.  Only oracle/ and synth/ are used.  The GPU test runs pahq_acdc_sweep with the same
receivers and thresholds and compares step by step.

  cfg2        restricted to six late receivers, a threshold that keeps edges
  cfg3        the three thresholds the config names, whole graph (on random-initialised weights each of
              them exceeds every increment: the pass removes the 157 in-edges of the output node and finds
              every other node dead)
  cfg3_keep   a threshold of 3e-4 (in a wide gap of the increments into the output node), restricted to the output node and three receivers of the
              top layer: a circuit with kept edges
  cfg4        the top MLP input of the config's seeded receiver sample at two thresholds: 1e-4 (above every
              increment: all 408 in-edges go, one by one, into an ever larger removed set) and 4e-5 (in the
              widest gap of those increments: edges are kept)

usage: python tests/golden/make_golden_sweep.py cfg2|cfg3|cfg3_keep|cfg4 [--resume]
  --resume    keep the runs an existing output file already holds for the same (threshold, receivers)
              (a run of config 4 takes more than an hour)
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


def runs_for(name, g, L, spec):
    top = L - 1
    if name == "cfg2":
        return "cfg2", [(5e-4, [g.OUT, g.mlpin(top), g.headin(top, 7, 2), g.headin(top, 7, 1), g.headin(top, 2, 0), g.headin(top - 1, 4, 2)])]
    if name == "cfg3":
        return "cfg3", [(tau, None) for tau in spec["taus"]]
    if name == "cfg3_keep":
        return "cfg3", [(3e-4, [g.OUT, g.mlpin(top), g.headin(top, 3, 1), g.headin(top, 7, 2)])]
    if name == "cfg4":
        sample = [int(r) for r in synth.make_receiver_sample(g.n_receivers, spec["n_recv"], spec["seed"])]
        assert g.mlpin(top) in sample
        return "cfg4", [(1e-4, [g.mlpin(top)]), (4e-5, [g.mlpin(top)])]
    raise SystemExit("no sweep defined for " + name)


def main():
    name = sys.argv[1]
    t0 = time.time()
    cfg = "cfg3" if name.startswith("cfg3") else name
    shape, w, clean, corrupt, spec = synth.make_workload(cfg)
    oa = Acdc(Model(shape, w), clean, corrupt)
    cfg, runs = runs_for(name, oa.g, shape.n_layers, spec)
    out = {"config": cfg, "seed": spec["seed"], "runs": []}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sweep_%s.json" % name)
    have = {}
    if "--resume" in sys.argv[2:] and os.path.exists(path):
        with open(path) as f:
            old = json.load(f)
        if old.get("config") == cfg and old.get("seed") == spec["seed"]:
            have = {(r["tau"], None if r["receivers"] is None else tuple(r["receivers"])): r for r in old["runs"]}
    for tau, recv in runs:
        key = (tau, None if recv is None else tuple(int(r) for r in recv))
        if key in have:
            out["runs"].append(have[key])
            print(name, "tau", tau, "kept from the existing file", flush=True)
            continue
        removed, trace = oa.sweep(tau, receivers=recv,
                                  progress=lambda v, n, r: print(name, "tau", tau, "receiver", v, "evals", n, "removed", r,
                                                                 "t=%.0fs" % (time.time() - t0), flush=True))
        out["runs"].append({"tau": tau, "receivers": None if recv is None else [int(r) for r in recv],
                            "trace": [[int(v), int(u), kn, kc, bool(rm)] for v, u, kn, kc, rm in trace],
                            "removed": [int(x) for x in oa.g.removed_to_flat(removed).nonzero()[0]]})
        print(name, "tau", tau, "evals", len(trace), "removed", len(out["runs"][-1]["removed"]), "t=%.0fs" % (time.time() - t0), flush=True)
        with open(path, "w") as f:
            json.dump(out, f)
    print("wrote", path, "in %.0f s" % (time.time() - t0))


if __name__ == "__main__":
    main()
