#!/usr/bin/env python3
"""Writes tests/golden/kl_<config>.json: per-edge KL values of the CPU oracle on a
seeded sample of candidates of one named config, at full size.

Only oracle/ and synth/ are used.  Each case is (receiver, removed-set recipe,
senders): the removed set is drawn with numpy default_rng(seed) as "each
in-edge of every receiver >= from_receiver removed with probability frac"
(frac = 0 gives the empty set), i.e. a state the sweep can be in when it
reaches that receiver.  The GPU tests rebuild the same workload and removed
sets and compare libpahq's pahq_eval_edges / pahq_eval_current against these
numbers.

usage: python tests/golden/make_golden_kl.py cfg3 [cfg4 ...]
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                   # noqa: E402
from oracle.model import Model                 # noqa: E402
from oracle.acdc import Acdc                   # noqa: E402


def removed_set(g, frac, seed, from_receiver):
    R = g.empty_removed()
    if frac <= 0:
        return R
    rng = np.random.default_rng(seed)
    for r in range(from_receiver, g.n_receivers):
        R[r, : g.n_upstream(r)] = rng.random(g.n_upstream(r)) < frac
    return R


def cases_for(name, g, L, H):
    """(receiver, frac, seed, senders) -- late layers for the large configs keep the oracle's cost bounded."""
    top = L - 1
    if name == "cfg3":
        return [(g.OUT, 0.0, 0, [0, 77, 156]), (g.OUT, 0.5, 1, [3, 100, 150]),
                (g.mlpin(top), 0.0, 0, [0, 140, 155]), (g.headin(top, 3, 1), 0.0, 0, [0, 90, 143]),
                (g.headin(8, 5, 2), 0.9, 2, [1, 50, 104]), (g.headin(6, 0, 0), 0.0, 0, [0, 40, 78]),
                (g.headin(9, 11, 1), 0.3, 3, [5, 60, 117])]
    if name == "cfg4":
        n = g.n_senders
        return [(g.OUT, 0.0, 0, [0, n // 2, n - 1]), (g.OUT, 0.9, 1, [7, n // 3, n - 2]),
                (g.mlpin(top), 0.0, 0, [0, n - 3]), (g.headin(top, 5, 1), 0.0, 0, [0, n // 2]),
                (g.headin(top - 1, 9, 2), 0.5, 2, [1, n // 2])]
    if name == "cfg5":
        n = g.n_senders
        return [(g.OUT, 0.0, 0, [0, n // 2, n - 1]), (g.mlpin(top), 0.0, 0, [0, n - 2]),
                (g.headin(top, 7, 1), 0.0, 0, [0, n // 2]), (g.headin(top, 20, 2), 0.9, 1, [3, n // 3])]
    raise SystemExit("no sample defined for " + name)


def main():
    for name in sys.argv[1:]:
        t0 = time.time()
        shape, w, clean, corrupt, spec = synth.make_workload(name)
        oa = Acdc(Model(shape, w, cache_decoded_bytes=2 << 30), clean, corrupt)
        g = oa.g
        out = {"config": name, "seed": spec["seed"], "mode": "PAHQ", "cases": []}
        for (r, frac, seed, senders) in cases_for(name, g, shape.n_layers, shape.n_heads):
            R = removed_set(g, frac, seed, r)
            cur = oa.kl_fast(r, R)
            kls = [oa.kl_edge(r, int(u), removed=R) for u in senders]
            out["cases"].append({"receiver": int(r), "frac": frac, "rseed": seed, "senders": [int(u) for u in senders],
                                 "kl_current": cur, "kl_new": kls})
            print(name, "receiver", r, "frac", frac, "cur", cur, "kl", kls, "t=%.0fs" % (time.time() - t0), flush=True)
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "kl_%s.json" % name)
        with open(path, "w") as f:
            json.dump(out, f, indent=1)
        print("wrote", path, "in %.0f s" % (time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
