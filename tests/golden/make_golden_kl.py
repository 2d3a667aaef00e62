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

usage: python tests/golden/make_golden_kl.py [--out-dir DIR] cfg3 [cfg4 cfg5_L2]
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
    """(receiver, frac, seed, number of senders) -- late layers for the large configs keep the
    oracle's cost bounded.  Senders are picked by pick_senders below."""
    top = L - 1
    if name == "cfg3":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.5, 1, 3), (g.mlpin(top), 0.0, 0, 3), (g.headin(top, 3, 1), 0.0, 0, 3),
                (g.headin(8, 5, 2), 0.9, 2, 2), (g.headin(6, 0, 0), 0.0, 0, 3), (g.headin(9, 11, 1), 0.3, 3, 2)]
    if name == "cfg4":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.9, 1, 3), (g.mlpin(top), 0.0, 0, 2), (g.headin(top, 5, 1), 0.0, 0, 2),
                (g.headin(top - 1, 9, 2), 0.5, 2, 2), (g.headin(top - 2, 0, 0), 0.0, 0, 2)]
    if name == "cfg5_L2":
        return [(g.OUT, 0.0, 0, 3), (g.OUT, 0.5, 1, 2), (g.mlpin(1), 0.0, 0, 3), (g.headin(1, 7, 1), 0.0, 0, 3),
                (g.headin(1, 20, 2), 0.5, 3, 2), (g.mlpin(0), 0.3, 2, 2), (g.headin(0, 31, 0), 0.0, 0, 1),
                (g.headin(0, 5, 2), 0.3, 4, 1)]
    raise SystemExit("no sample defined for " + name)


def pick_senders(R, r, n_up, k):
    """k kept senders spread over the kept in-edges of r (first, ..., last), plus one already
    removed sender when there is one (its candidate equals the current state)."""
    kept = np.flatnonzero(~R[r, :n_up])
    rem = np.flatnonzero(R[r, :n_up])
    picks = [int(kept[i]) for i in np.unique(np.linspace(0, len(kept) - 1, k).round().astype(int))] if len(kept) else []
    if len(rem):
        picks.append(int(rem[len(rem) // 2]))
    return picks


def main():
    args = sys.argv[1:]
    out_dir = os.path.dirname(os.path.abspath(__file__))
    if args and args[0] == "--out-dir":
        out_dir = args[1]
        args = args[2:]
        os.makedirs(out_dir, exist_ok=True)
    for name in args:
        t0 = time.time()
        shape, w, clean, corrupt, spec = synth.make_workload(name)
        print(name, "workload made t=%.0fs" % (time.time() - t0), flush=True)
        oa = Acdc(Model(shape, w, cache_decoded_bytes=2 << 30), clean, corrupt)
        g = oa.g
        print(name, "weights quantised t=%.0fs" % (time.time() - t0), flush=True)
        out = {"config": name, "seed": spec["seed"], "mode": "PAHQ", "cases": []}
        for (r, frac, seed, k) in cases_for(name, g, shape.n_layers, shape.n_heads):
            R = removed_set(g, frac, seed, r)
            senders = pick_senders(R, r, g.n_upstream(r), k)
            cur = oa.kl_fast(r, R)
            print(name, "receiver", r, "current state done t=%.0fs" % (time.time() - t0), flush=True)
            kls = []
            for u in senders:
                kls.append(oa.kl_edge(r, int(u), removed=R))
                print(name, "receiver", r, "sender", u, "done t=%.0fs" % (time.time() - t0), flush=True)
            out["cases"].append({"receiver": int(r), "frac": frac, "rseed": seed, "senders": [int(u) for u in senders],
                                 "kl_current": cur, "kl_new": kls})
            print(name, "receiver", r, "frac", frac, "cur", cur, "kl", kls, "t=%.0fs" % (time.time() - t0), flush=True)
        path = os.path.join(out_dir, "kl_%s.json" % name)
        with open(path, "w") as f:
            json.dump(out, f, indent=1)
        print("wrote", path, "in %.0f s" % (time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
