"""Host-resident fp32 masters with prefetch (pahq_config.fp32_residency = PAHQ_FP32_ON_HOST) against the default,
where every master lives in the workspace.

Paper, Sec. "Selective Precision Allocation Strategy" (Hierarchical Weight Scheduling: the fp32 weights of S_t must
be on the device at step t, those of S_t+1 are moved while step t computes) and Sec. "Algorithm Implementation in
Practice" (Scheduler Implementation).  Where the weights come from changes no arithmetic, so every result of the
two models must agree bit for bit -- weight codes (the masters reach the quantiser through a staging buffer), cache
passes, per-edge values in any order, sweeps, circuit evaluations with arbitrary sets of fp32 heads -- and parity with
the oracle then follows from the default model's.  The transfer counters must show that in sweep order only the
first joint pass of a layer's heads waits for its weights.
"""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402
from oracle.graph import Graph                      # noqa: E402
from test_gpu_parity import random_removed          # noqa: E402

pytestmark = pytest.mark.gpu


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def pair(P, name, **kw):
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    a = P.Model(shape, w, B, S, max_batch_edges=8, **kw)
    b = P.Model(shape, w, B, S, max_batch_edges=8, fp32_on_host=True, **kw)
    return shape, clean, corrupt, a, b


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi", "cfg1_hi"])
def test_results_are_bit_identical(name):
    import paper_2510_23264_amd as P
    shape, clean, corrupt, a, b = pair(P, name)
    L, H, dh, d, m = shape.n_layers, shape.n_heads, shape.d_head, shape.d_model, shape.d_mlp
    g = Graph(L, H, m > 0)
    try:
        if L > 2:          # the device keeps two layers' worth of head slots and one staging buffer
            assert b.workspace_bytes < a.workspace_bytes
        # weight codes and scales: every class, first and last layer
        for l in (0, L - 1):
            for which, sh in ((0, (d, dh)), (2, (d, dh)), (3, (dh, d))):        # PAHQ_W_Q, PAHQ_W_V, PAHQ_W_O
                for h in (0, H - 1):
                    ca, sa = a.get_weight_q(which, l, h, sh)
                    cb, sb = b.get_weight_q(which, l, h, sh)
                    assert np.array_equal(ca, cb) and sa == sb, (name, which, l, h)
            if m > 0:
                for which, sh in ((4, (d, m)), (6, (m, d))):
                    ca, sa = a.get_weight_q(which, l, 0, sh)
                    cb, sb = b.get_weight_q(which, l, 0, sh)
                    assert np.array_equal(ca, cb) and sa == sb, (name, which, l)
        ca, sa = a.get_weight_q(7, 0, 0, (d, shape.vocab))
        cb, sb = b.get_weight_q(7, 0, 0, (d, shape.vocab))
        assert np.array_equal(ca, cb) and sa == sb
        for gm in (a, b):
            gm.clean_cache(clean, corrupt)
        assert np.array_equal(bits(a.get_logits(0)), bits(b.get_logits(0)))
        assert np.array_equal(bits(a.get_sender_output(0, g.n_senders - 1)), bits(b.get_sender_output(0, g.n_senders - 1)))
        # per-edge values: receivers in ASCENDING order (against the prediction), then a random order, at the empty set
        recvs = list(range(g.n_receivers))
        rng = np.random.default_rng(11)
        for order in (recvs, list(rng.permutation(recvs)[:12])):
            for r in order:
                s = np.arange(g.n_upstream(r), dtype=np.int32)
                assert np.array_equal(bits(a.eval_edges(r, s)), bits(b.eval_edges(r, s))), (name, r)
                assert a.eval_current(r) == b.eval_current(r)
        # a pruned state (slots, kept forms, dead nodes), edge lists over a whole layer
        r0 = g.headin(L - 1, 0, 0)
        R = g.removed_to_flat(random_removed(g, 0.6, 5, from_receiver=r0)).astype(np.uint8)
        rr = np.concatenate([np.full(g.n_upstream(r), r, np.int32) for r in range(r0, r0 + 3 * H)])
        ss = np.concatenate([np.arange(g.n_upstream(r), dtype=np.int32) for r in range(r0, r0 + 3 * H)])
        for gm in (a, b):
            gm.set_removed(R)
        assert np.array_equal(bits(a.eval_edge_list(rr, ss)), bits(b.eval_edge_list(rr, ss)))
        # circuit evaluation under sets of fp32 heads: none, one, every second layer, random, all
        sets = [np.zeros((L, H), np.uint8), np.ones((L, H), np.uint8), (rng.random((L, H)) < 0.5).astype(np.uint8)]
        one = np.zeros((L, H), np.uint8); one[L - 1, H - 1] = 1; sets.append(one)
        alt = np.zeros((L, H), np.uint8); alt[::2] = 1; sets.append(alt)
        kept = (rng.random(g.n_edges()) < 0.7).astype(np.uint8)
        for f in sets:
            ka, la = a.eval_circuit(kept=kept, f32_heads=f, want_logits=True)
            kb, lb = b.eval_circuit(kept=kept, f32_heads=f, want_logits=True)
            assert ka == kb and np.array_equal(bits(la), bits(lb)), (name, f.sum())
    finally:
        a.close(); b.close()


@pytest.mark.parametrize("name", ["mid_hi", "cfg1_hi"])
def test_sweeps_are_identical_and_transfers_run_ahead(name):
    import paper_2510_23264_amd as P
    shape, clean, corrupt, a, b = pair(P, name)
    L, H = shape.n_layers, shape.n_heads
    try:
        for gm in (a, b):
            gm.clean_cache(clean, corrupt)
        s0 = b.transfer_stats()
        assert s0["head_uses"] == 0 and s0["bytes_moved"] == 0            # the cache passes have no fp32 head
        head_bytes = s0["slot_bytes"] // (2 * H)
        assert s0["host_bytes"] == L * H * head_bytes
        for tau in (1e-3, -1.0):                  # the second removes nothing: every edge is evaluated, in order
            before = b.transfer_stats()
            ka, na, ta = a.acdc_sweep(tau)
            kb, nb, tb = b.acdc_sweep(tau)
            assert na == nb and np.array_equal(ka, kb)
            assert ta.tobytes() == tb.tobytes(), (name, tau)
            s1 = b.transfer_stats()
            assert s1["head_uses"] > before["head_uses"]
            assert s1["bytes_moved"] == (s1["demand_transfers"] + s1["transfers_ahead"]) * head_bytes
            if kb.all():
                # nothing was removed, so no receiver was skipped and the sweep met every head in the predicted order:
                # only the top layer's first pass found nothing on the device
                assert s1["demand_transfers"] - before["demand_transfers"] <= H, (before, s1)
                # ... every other head arrived ahead of its use or was still there from the sweep before, and none
                # moved twice
                moved = (s1["bytes_moved"] - before["bytes_moved"]) // head_bytes
                assert moved <= L * H, (before, s1)
                if L > 2:
                    assert s1["transfers_ahead"] - before["transfers_ahead"] >= H, (before, s1)
        # the sender-side policy (fp32 for the edge's source head) takes its weights on demand: same decisions
        if L * H <= 16:
            ka, na, ta = a.acdc_sweep(1e-4, sender_policy=True)
            kb, nb, tb = b.acdc_sweep(1e-4, sender_policy=True)
            assert na == nb and np.array_equal(ka, kb) and ta.tobytes() == tb.tobytes()
    finally:
        a.close(); b.close()


def test_prefetch_hints_and_errors():
    import paper_2510_23264_amd as P
    shape, clean, corrupt, a, b = pair(P, "mid_hi")
    L, H = shape.n_layers, shape.n_heads
    g = Graph(L, H, shape.d_mlp > 0)
    try:
        with pytest.raises(P.PahqError):
            a.prefetch_heads(0, [0])                   # not a host-resident model
        with pytest.raises(P.PahqError):
            a.transfer_stats()
        with pytest.raises(P.PahqError):
            b.prefetch_heads(L, [0])
        if H < 64:
            with pytest.raises(P.PahqError):
                b.prefetch_heads(0, [H])
        for gm in (a, b):
            gm.clean_cache(clean, corrupt)
        # right hints: no demand transfer at all; wrong hints (other heads, heads that share the slot of the one
        # needed) cost a wait and nothing else
        r = g.headin(0, 0, 1)
        s = np.arange(g.n_upstream(r), dtype=np.int32)
        b.prefetch_heads(0, range(H))
        want = a.eval_edges(r, s)
        assert np.array_equal(bits(b.eval_edges(r, s)), bits(want))
        assert b.transfer_stats()["demand_transfers"] == 0
        for it in range(3):
            if L > 2:
                b.prefetch_heads(2, [0])               # same slot as head (0, 0)
            b.prefetch_heads(L - 1, [H - 1])
            assert np.array_equal(bits(b.eval_edges(r, s)), bits(want))
        r2 = g.headin(L - 1, H - 1, 2)
        s2 = np.arange(g.n_upstream(r2), dtype=np.int32)
        assert np.array_equal(bits(b.eval_edges(r2, s2)), bits(a.eval_edges(r2, s2)))
    finally:
        a.close(); b.close()


@pytest.mark.parametrize("opts", [dict(low_bits=16), dict(nonattn_bf16=True), dict(split_qkv=False), dict(low_bits=4),
                                  dict(precision="all_fp8")])
def test_composes_with_the_other_options(opts):
    import paper_2510_23264_amd as P
    opts = dict(opts)
    if opts.get("precision") == "all_fp8":
        opts["precision"] = P.ALL_FP8
    shape, clean, corrupt, a, b = pair(P, "mid_hi", **opts)
    L, H = shape.n_layers, shape.n_heads
    try:
        for gm in (a, b):
            gm.clean_cache(clean, corrupt)
        ka, na, ta = a.acdc_sweep(1e-4)
        kb, nb, tb = b.acdc_sweep(1e-4)
        assert na == nb and np.array_equal(ka, kb) and ta.tobytes() == tb.tobytes(), opts
        f = (np.random.default_rng(3).random((L, H)) < 0.5).astype(np.uint8)
        assert a.eval_circuit(kept=ka, f32_heads=f) == b.eval_circuit(kept=kb, f32_heads=f)
        if opts.get("precision") == P.ALL_FP8:
            assert b.transfer_stats()["bytes_moved"] == 0 or f.any()
    finally:
        a.close(); b.close()


def test_all_fp32_refuses_host_residency():
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make("mid_hi")
    with pytest.raises(P.PahqError):
        P.Model(shape, w, clean.shape[0], clean.shape[1], precision=P.ALL_FP32, fp32_on_host=True)


def test_config3_shape_edge_lists_and_restricted_sweep():
    """The GPT-2-small shape: a layer's edge list and a sweep over the output node and the two top layers, bit for bit
    against the resident model, with every head's weights arriving ahead of its use."""
    import synth
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt, spec = synth.make_workload("cfg3")
    B, S = spec["B"], spec["S"]
    L, H = shape.n_layers, shape.n_heads
    a = P.Model(shape, w, B, S, max_batch_edges=32)
    b = P.Model(shape, w, B, S, max_batch_edges=32, fp32_on_host=True)
    try:
        assert a.workspace_bytes - b.workspace_bytes > 300e6          # the fp32 matrix masters less the slots and the staging buffer
        for gm in (a, b):
            gm.clean_cache(clean, corrupt)
        per_layer = 3 * H + 1
        recvs = list(range((L - 1) * per_layer, L * per_layer))[::-1]
        rr = np.concatenate([np.full(P.n_upstream(a.cfg, r), r, np.int32) for r in recvs])[::3]
        ss = np.concatenate([np.arange(P.n_upstream(a.cfg, r), dtype=np.int32) for r in recvs])[::3]
        b.prefetch_heads(L - 1, range(H))
        assert np.array_equal(bits(a.eval_edge_list(rr, ss)), bits(b.eval_edge_list(rr, ss)))
        assert b.transfer_stats()["demand_transfers"] == 0
        top = np.arange((L - 2) * per_layer, L * per_layer + 1, dtype=np.int32)
        ka, na, ta = a.acdc_sweep(1e-4, receivers=top)
        kb, nb, tb = b.acdc_sweep(1e-4, receivers=top)
        assert na == nb and np.array_equal(ka, kb) and ta.tobytes() == tb.tobytes()
        st = b.transfer_stats()
        assert st["demand_transfers"] <= H and st["transfers_ahead"] >= H, st
    finally:
        a.close(); b.close()
