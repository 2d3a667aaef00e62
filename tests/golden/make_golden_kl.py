#!/usr/bin/env python3
"""Writes tests/golden/kl_<workload>.json: per-edge KL values of the CPU oracle on a seeded sample of
candidates of one workload of tests/golden/workloads.py, with the spread binary32 arithmetic leaves in
each value (tests/fp32_spread.py).

Only oracle/, synth/ and the two test-side modules named above are used.  Each case is (receiver,
removed-set recipe, senders).  The GPU tests rebuild the same workload and removed sets and compare
libpahq's pahq_eval_edges / pahq_eval_current against these numbers.

usage: python tests/golden/make_golden_kl.py [--out-dir DIR] [--seeds N] workload [workload ...]
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)

from oracle.acdc import MODE_PAHQ                 # noqa: E402
from fp32_spread import SpreadModel, kl_with_spread, EPS   # noqa: E402
import workloads                                  # noqa: E402

DEFAULT_SEEDS = {"cfg1_hi": 8, "mid_hi": 8, "mid_hi2": 8, "midllama_hi": 8, "midllama_hi2": 8, "cfg2": 4, "cfg2_hi": 4}


def pick_senders(row, k):
    """k kept senders spread over the kept in-edges (first, ..., last), plus one already removed sender
    when there is one (its candidate equals the current state).  k = 0: every sender."""
    if k == 0:
        return list(range(len(row)))
    kept, rem = np.flatnonzero(~row), np.flatnonzero(row)
    picks = [int(kept[i]) for i in np.unique(np.linspace(0, len(kept) - 1, k).round().astype(int))] if len(kept) else []
    if len(rem):
        picks.append(int(rem[len(rem) // 2]))
    return picks


def case_list(name, g, L, H):
    """(receiver, frac, seed, number of senders; 0 = all).  Late layers for the large shapes keep the
    oracle's cost bounded."""
    top = L - 1
    if name in ("cfg1_hi",):
        return [(r, 0.0, 0, 0) for r in range(g.n_receivers)] + [(r, 0.5, 100 + r, 0) for r in (g.OUT, g.n_receivers // 2, 1)]
    if name in ("mid_hi", "mid_hi2", "midllama_hi", "midllama_hi2"):
        return [(r, 0.0, 0, 0) for r in range(g.n_receivers - 1, -1, -3)] + \
               [(r, 0.5, 100 + r, 0) for r in (g.OUT, g.mlpin(top), g.headin(top, 1, 1), g.headin(1, 0, 2), g.mlpin(0), 1)]
    if name in ("cfg2", "cfg2_hi"):
        return [(g.OUT, 0.0, 0, 6), (g.OUT, 0.5, 1, 4), (g.mlpin(3), 0.0, 0, 4), (g.headin(3, 0, 1), 0.0, 0, 4),
                (g.headin(3, 5, 2), 0.5, 2, 3), (g.headin(2, 1, 2), 0.0, 0, 4), (g.mlpin(1), 0.3, 3, 3),
                (g.headin(1, 0, 0), 0.0, 0, 4), (g.mlpin(0), 0.0, 0, 2)]
    if name == "cfg3":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.5, 1, 3), (g.mlpin(top), 0.0, 0, 3), (g.headin(top, 3, 1), 0.0, 0, 3),
                (g.headin(8, 5, 2), 0.9, 2, 2), (g.headin(6, 0, 0), 0.0, 0, 3), (g.headin(9, 11, 1), 0.3, 3, 2)]
    if name == "cfg3_hi":
        return [(g.OUT, 0.0, 0, 4), (g.OUT, 0.5, 1, 3), (g.mlpin(top), 0.0, 0, 3), (g.headin(top, 3, 1), 0.5, 4, 3),
                (g.headin(9, 11, 1), 0.0, 0, 3), (g.headin(8, 5, 2), 0.9, 2, 2)]
    if name == "cfg4":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.9, 1, 3), (g.mlpin(top), 0.0, 0, 2), (g.headin(top, 5, 1), 0.0, 0, 2),
                (g.headin(top - 1, 9, 2), 0.5, 2, 2), (g.headin(top - 2, 0, 0), 0.0, 0, 2)]
    if name == "cfg5_L2":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.5, 1, 2), (g.mlpin(1), 0.0, 0, 3), (g.headin(1, 7, 1), 0.0, 0, 3),
                (g.headin(1, 20, 2), 0.5, 3, 2), (g.mlpin(0), 0.3, 2, 2), (g.headin(0, 31, 0), 0.0, 0, 1),
                (g.headin(0, 5, 2), 0.3, 4, 1)]
    if name == "cfg5_L8":
        return [(g.OUT, 0.0, 0, 2), (g.OUT, 0.5, 1, 1), (g.headin(top, 20, 1), 0.0, 0, 2), (g.mlpin(top - 1), 0.3, 2, 1)]
    raise SystemExit("no sample defined for " + name)


def main():
    args = sys.argv[1:]
    out_dir, seeds_arg = HERE, None
    while args and args[0].startswith("--"):
        if args[0] == "--out-dir":
            out_dir = args[1]
            os.makedirs(out_dir, exist_ok=True)
        elif args[0] == "--seeds":
            seeds_arg = int(args[1])
        else:
            raise SystemExit("unknown option " + args[0])
        args = args[2:]
    for name in args:
        t0 = time.time()
        shape, w, clean, corrupt = workloads.make(name)
        print(name, "workload made t=%.0fs" % (time.time() - t0), flush=True)
        om = SpreadModel(shape, w, cache_decoded_bytes=2 << 30)
        g = om.g
        print(name, "weights quantised t=%.0fs" % (time.time() - t0), flush=True)
        seeds = seeds_arg if seeds_arg is not None else DEFAULT_SEEDS.get(name, 3)
        specs, cases = case_list(name, g, shape.n_layers, shape.n_heads), []
        for (r, frac, rseed, k) in specs:
            rows = workloads.removed_rows(g.n_receivers, g.n_upstream, frac, rseed, r)
            R = g.empty_removed()
            for q, row in enumerate(rows):
                R[q, :len(row)] = row
            cases.append((r, R, pick_senders(rows[r], k)))
        res = kl_with_spread(om, clean, corrupt, MODE_PAHQ, cases, seeds=seeds,
                             progress=lambda r: print(name, "receiver", r, "done t=%.0fs" % (time.time() - t0), flush=True))
        out = {"workload": name, "mode": "PAHQ", "spread_eps": EPS, "spread_seeds": seeds, "cases": []}
        for (r, frac, rseed, k), (_, _, senders), o in zip(specs, cases, res):
            out["cases"].append({"receiver": int(r), "frac": frac, "rseed": rseed, "senders": [int(u) for u in senders], **o})
        path = os.path.join(out_dir, "kl_%s.json" % name)
        with open(path, "w") as f:
            json.dump(out, f, indent=None if len(out["cases"]) > 12 else 1)
        kls = np.array([k for c in out["cases"] for k in c["kl_new"]])
        print("wrote", path, "in %.0f s: %d values, median KL %.3g, max %.3g" % (time.time() - t0, kls.size, np.median(kls), kls.max()), flush=True)


if __name__ == "__main__":
    main()
