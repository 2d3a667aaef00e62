"""GPU parity at the full sizes of the named configs, on sampled candidates.

Expected values come from tests/golden/kl_<config>.json, written by
tests/golden/make_golden_kl.py (CPU oracle only).  Each case fixes a receiver,
a seeded removed set (a state the sweep can be in when it reaches that
receiver) and a few senders; the device evaluates exactly these through the C
ABI, in the launch configuration bench.py uses (e4m3 operands with exact fp32
sums, batch 128).  The FP8 matrix-core instruction is run as well: its adder
truncates products against the largest one of an instruction, which makes
every KL come out about 1.3 % low (measured); that mode is held to
1e-4 + 2.5e-2 |KL| and is not the default."""
import json
import os
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KL_ATOL, KL_RTOL = 1e-4, 1e-3


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


def run_config(name, max_batch, mma=1, rtol=KL_RTOL):
    import paper_2510_23264_amd as P
    path = os.path.join(GOLDEN, "kl_%s.json" % name)
    if not os.path.exists(path):
        pytest.skip("no golden file for " + name)
    gold = json.load(open(path))
    shape, w, clean, corrupt, spec = synth.make_workload(name)
    assert spec["seed"] == gold["seed"]
    gm = P.Model(shape, w, spec["B"], spec["S"], precision=P.PAHQ, max_batch_edges=max_batch, mma=mma)
    try:
        gm.clean_cache(clean, corrupt)
        worst = 0.0
        for case in gold["cases"]:
            r = case["receiver"]
            gm.set_removed(removed_flat(gm.cfg, P, case["frac"], case["rseed"], r))
            cur = gm.eval_current(r)
            assert abs(cur - case["kl_current"]) <= KL_ATOL + rtol * abs(case["kl_current"]), (name, r, cur, case["kl_current"])
            got = gm.eval_edges(r, np.array(case["senders"], np.int32))
            for u, g_, want in zip(case["senders"], got, case["kl_new"]):
                tol = KL_ATOL + rtol * abs(want)
                assert abs(g_ - want) <= tol, (name, r, u, float(g_), want)
                worst = max(worst, abs(g_ - want) / (KL_ATOL + KL_RTOL * abs(want)))
        print(name, "worst |d| / (1e-4 + 1e-3 |KL|) =", worst)
    finally:
        gm.close()


def test_cfg3_sampled_edges():
    run_config("cfg3", 128)


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


def test_cfg3_sampled_edges_fp8_matrix_core_adder():
    run_config("cfg3", 64, mma=0, rtol=2.5e-2)


def test_cfg4_sampled_edges():
    run_config("cfg4", 16)


def test_cfg5_layer_shape_depth2_sampled_edges():
    """Config 5's layer shape, batch and token recipe at depth 2 (the CPU check of 32 such
    layers takes hours): every kernel shape config 5 launches, against the CPU values.

    Held to 1e-4 + 2e-3 |KL|, twice the relative part of the tolerance used elsewhere, and the
    worst ratio against the usual tolerance is printed (measured: 1.5).  At d_model 4096 /
    d_mlp 11008 the binary32 sums of the device and the fp64 sums of the CPU model differ by
    about 1e-6 relative per GEMM output; each such difference that straddles an e4m3 rounding
    boundary moves one code by a whole step (2^-4 relative), and a layer has millions of
    outputs.  The resulting KL differences have both signs and about 1e-3 relative size: they
    are the quantiser's discontinuity, not a bias (the FP8 matrix-core adder, which is biased,
    shows up as 1.3 % on every candidate)."""
    run_config("cfg5_L2", 8, rtol=2e-3)


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


def test_cfg2_restricted_sweep_matches_oracle_trace():
    """pahq_acdc_sweep restricted to a few receivers of config 2 against the oracle's literal
    one-by-one pass (tests/golden/sweep_cfg2.json).  A decision may differ only where the KL
    increment lies within the tolerance of tau; the comparison stops there because every
    later state differs."""
    import paper_2510_23264_amd as P
    path = os.path.join(GOLDEN, "sweep_cfg2.json")
    if not os.path.exists(path):
        pytest.skip("no golden sweep for cfg2")
    gold = json.load(open(path))
    shape, w, clean, corrupt, spec = synth.make_workload("cfg2")
    for mma in (P.MMA_F16_EXACT,):
        gm = P.Model(shape, w, spec["B"], spec["S"], max_batch_edges=16, mma=mma)
        try:
            gm.clean_cache(clean, corrupt)
            kept, n_evals, tr = gm.acdc_sweep(gold["tau"], receivers=np.array(gold["receivers"], np.int32))
            diverged = False
            for i, (v, u, kn, kc, rm) in enumerate(gold["trace"]):
                if i >= n_evals:
                    break
                t = tr[i]
                assert (t["receiver"], t["sender"]) == (v, u), (mma, i)
                assert abs(t["kl_new"] - kn) <= KL_ATOL + KL_RTOL * abs(kn), (mma, i, t, kn)
                assert abs(t["kl_cur"] - kc) <= KL_ATOL + KL_RTOL * abs(kc), (mma, i, t, kc)
                if bool(t["removed"]) != rm:
                    assert abs((kn - kc) - gold["tau"]) <= 2 * (KL_ATOL + KL_RTOL * abs(kn)), (mma, i, t, kn, kc)
                    diverged = True
                    break
            if not diverged:
                assert n_evals == len(gold["trace"])
                removed = np.flatnonzero(kept == 0)
                assert removed.tolist() == gold["removed"]
        finally:
            gm.close()
