"""GPU tests at the full sizes of the named configs that need no per-candidate oracle value (batch
invariance, properties that hold at any size) and the sweeps against stored oracle traces.  Sampled
per-edge values are compared in tests/test_gpu_golden.py."""
import json
import os
import numpy as np
import pytest

import synth
from tolerance import north_star, bound, pooled

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def removed_flat(cfg, P, frac, seed, from_receiver):
    """Same recipe as make_golden_kl.removed_set, in canonical edge order."""
    n_recv = P.n_receivers(cfg)
    parts = []
    rng = np.random.default_rng(seed)
    for r in range(n_recv):
        n_up = P.n_upstream(cfg, r)
        if frac > 0 and r >= from_receiver:
            parts.append((rng.random(n_up) < frac).astype(np.uint8))
        else:
            parts.append(np.zeros(n_up, np.uint8))
    return np.concatenate(parts)


def test_cfg3_gather_with_most_edges_removed_is_batch_invariant():
    """With 90 % of the edges removed a receiver's input is gathered from many terms, most of them tiles every
    candidate shares; a full batch takes the kernel that sums those once for a chunk of instances, a batch of one
    does not chunk.  The KL of a candidate has the same bits either way, also against the current state when the
    candidate's edge is already removed."""
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt, spec = synth.make_workload("cfg3")
    gm = P.Model(shape, w, spec["B"], spec["S"], precision=P.PAHQ, max_batch_edges=128)
    try:
        gm.clean_cache(clean, corrupt)
        n_recv = P.n_receivers(gm.cfg)
        r = n_recv // 2                       # a receiver in the middle of the model: six layers are recomputed
        removed = removed_flat(gm.cfg, P, 0.9, 77, r)
        gm.set_removed(removed)
        n_up = P.n_upstream(gm.cfg, r)
        senders = np.arange(n_up, dtype=np.int32)[:128]
        batch = gm.eval_edges(r, senders)
        ones = np.array([gm.eval_edges(r, senders[i:i + 1])[0] for i in range(0, senders.size, 9)], np.float32)
        assert (ones.view(np.uint32) == batch[::9].view(np.uint32)).all()
        off = int(sum(P.n_upstream(gm.cfg, q) for q in range(r)))
        gone = [int(u) for u in senders if removed[off + int(u)]]
        assert gone
        cur = np.float32(gm.eval_current(r))
        assert all(np.float32(batch[u]).view(np.uint32) == cur.view(np.uint32) for u in gone)
    finally:
        gm.close()


@pytest.mark.timeout(1000)
def test_cfg5_full_size_properties():
    """Config 5 at full depth, through properties that need no CPU value: the clean run
    patched with nothing has KL exactly 0; a candidate whose edge is already removed equals
    the current state bit for bit; results do not depend on how candidates are batched;
    removing edges moves the KL away from 0 and never gives NaN."""
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt, spec = synth.make_workload("cfg5")
    print("cfg5: weights drawn", flush=True)
    gm = P.Model(shape, w, spec["B"], spec["S"], precision=P.PAHQ, max_batch_edges=8)
    try:
        del w
        print("cfg5: model on the device", flush=True)
        gm.clean_cache(clean, corrupt)
        print("cfg5: caches filled", flush=True)
        from oracle.graph import Graph
        g = Graph(shape.n_layers, shape.n_heads, shape.d_mlp > 0)
        out_r = g.OUT
        top = shape.n_layers - 1
        key_r = g.headin(top, 20, 1)
        for r in (out_r, key_r):
            assert gm.eval_current(r) == 0.0
        n_up = P.n_upstream(gm.cfg, out_r)
        senders = np.array([0, 1, n_up // 2, n_up - 2, n_up - 1], np.int32)
        a = gm.eval_edges(out_r, senders)
        assert np.isfinite(a).all() and a[0] == 0.0 and (a[1:] > 0).all()       # EMBED -> OUT: same tokens
        one = np.array([gm.eval_edges(out_r, senders[i:i + 1])[0] for i in range(len(senders))])
        assert np.array_equal(a, one)
        rem = removed_flat(gm.cfg, P, 0.5, 1, key_r)
        gm.set_removed(rem)
        cur = gm.eval_current(key_r)
        assert np.isfinite(cur) and cur > 0
        off = int(g.edge_offsets()[key_r])
        nk = P.n_upstream(gm.cfg, key_r)
        gone = np.flatnonzero(rem[off:off + nk])[:2].astype(np.int32)
        kept = np.flatnonzero(rem[off:off + nk] == 0)[:3].astype(np.int32)
        got = gm.eval_edges(key_r, np.concatenate([gone, kept]))
        assert got[0] == cur and got[1] == cur
        assert np.isfinite(got).all()
        again = gm.eval_edges(key_r, kept[::-1].copy())
        assert np.array_equal(again[::-1], got[2:])
    finally:
        gm.close()


def pooled_increment_spread(name):
    """rms over the stored cases of a workload of the spread binary32 arithmetic leaves in an increment
    (0 where the stored values carry none: the bound is then the tight one)."""
    gold = json.load(open(os.path.join(GOLDEN, "kl_%s.json" % name)))
    if "spread_eps" not in gold:
        return 0.0
    return pooled([v for c in gold["cases"] for v in c["sigma_inc"]])


@pytest.mark.parametrize("name,batch", [("cfg2", 16), ("cfg3", 128), ("cfg3_keep", 128), ("cfg4", 16)])
def test_sweep_matches_the_oracle_trace(name, batch):
    """pahq_acdc_sweep against the oracle's literal one-by-one pass (tests/golden/sweep_<name>.json,
    written by make_golden_sweep.py): the trace step by step, then the kept set.  A decision may differ
    only where the oracle's increment lies within the parity bound of tau (tests/tolerance.py, with the
    workload's pooled increment spread); the comparison stops there because every later state differs."""
    import paper_2510_23264_amd as P
    path = os.path.join(GOLDEN, "sweep_%s.json" % name)
    if not os.path.exists(path):
        pytest.skip("no stored sweep for " + name)
    gold = json.load(open(path))
    cfg_name = gold["config"]
    shape, w, clean, corrupt, spec = synth.make_workload(cfg_name)
    spread = pooled_increment_spread(cfg_name)
    gm = P.Model(shape, w, spec["B"], spec["S"], max_batch_edges=batch)
    try:
        del w
        gm.clean_cache(clean, corrupt)
        for run in gold["runs"]:
            tau = run["tau"]
            recv = None if run["receivers"] is None else np.array(run["receivers"], np.int32)
            kept, n_evals, tr = gm.acdc_sweep(tau, receivers=recv)
            diverged = False
            for i, (v, u, kn, kc, rm) in enumerate(run["trace"]):
                if i >= n_evals:
                    break
                t = tr[i]
                assert (t["receiver"], t["sender"]) == (v, u), (name, tau, i)
                assert abs(t["kl_new"] - kn) <= north_star(kn), (name, tau, i, t, kn)
                assert abs(t["kl_cur"] - kc) <= north_star(kc), (name, tau, i, t, kc)
                if bool(t["removed"]) != rm:
                    assert abs((kn - kc) - tau) <= bound(max(abs(kn), abs(kc)), spread), (name, tau, i, t, kn, kc)
                    diverged = True
                    break
            if not diverged:
                assert n_evals == len(run["trace"]), (name, tau)
                assert np.flatnonzero(kept == 0).tolist() == run["removed"], (name, tau)
            print(name, "tau", tau, "diverged inside the bound at step %d" % i if diverged else "equal",
                  "evals", n_evals, "kept", int(kept.sum()))
    finally:
        gm.close()
