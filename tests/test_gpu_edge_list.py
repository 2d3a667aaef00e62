"""pahq_eval_edge_list against pahq_eval_edges: the same values bit for bit, whatever the order of the list
and however its runs are cut into device batches, with fewer batches where the query, key and value inputs
of a head share them."""
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


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi", "cfg1_hi"])
@pytest.mark.parametrize("mode", ["pahq", "all_fp8"])
def test_edge_list_equals_per_receiver_calls(name, mode):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    g = Graph(shape.n_layers, shape.n_heads, shape.d_mlp > 0)
    gm = P.Model(shape, w, B, S, precision=P.PAHQ if mode == "pahq" else P.ALL_FP8, max_batch_edges=8)
    try:
        gm.clean_cache(clean, corrupt)
        rng = np.random.default_rng(4)
        for state in ("empty", "pruned"):
            if state == "empty":
                recvs = list(range(g.n_receivers))
            else:
                r0 = g.headin(shape.n_layers - 1, 0, 0)
                gm.set_removed(g.removed_to_flat(random_removed(g, 0.5, 6, from_receiver=r0)).astype(np.uint8))
                recvs = list(range(r0 + 3 * shape.n_heads))          # every receiver up to and including r0's layer inputs
            per = {r: gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) for r in recvs}
            b0 = gm.counters()[1]
            rr = np.concatenate([np.full(g.n_upstream(r), r, np.int32) for r in recvs])
            ss = np.concatenate([np.arange(g.n_upstream(r), dtype=np.int32) for r in recvs])
            want = np.concatenate([per[r] for r in recvs])
            got = gm.eval_edge_list(rr, ss)
            b_list = gm.counters()[1] - b0
            assert np.array_equal(bits(got), bits(want)), (name, mode, state, np.argwhere(bits(got) != bits(want))[:5].ravel())
            b_per = sum(-(-g.n_upstream(r) // 8) for r in recvs)
            if mode == "pahq":
                assert b_list < b_per, (b_list, b_per)               # the three inputs of a head share batches
            # any order: receivers descending (value, key, query: no sharing, still the same values) ...
            order = np.argsort(-rr, kind="stable")
            assert np.array_equal(bits(gm.eval_edge_list(rr[order], ss[order])), bits(want[order]))
            # ... a random permutation (runs of length one), a subset with repeats
            perm = rng.permutation(len(rr))[:200]
            perm = np.concatenate([perm, perm[:7]])
            assert np.array_equal(bits(gm.eval_edge_list(rr[perm], ss[perm])), bits(want[perm]))
            # ... and partial runs: two of a head's three inputs, some senders of each
            h_in = [g.headin(shape.n_layers - 1, 1 % shape.n_heads, c) for c in (0, 2)]
            sel = np.concatenate([np.flatnonzero((rr == r) & (ss % 2 == i)) for i, r in enumerate(h_in)])
            assert np.array_equal(bits(gm.eval_edge_list(rr[sel], ss[sel])), bits(want[sel]))
        assert gm.eval_edge_list(np.zeros(0, np.int32), np.zeros(0, np.int32)).size == 0
        with pytest.raises(P.PahqError):
            gm.eval_edge_list(np.array([g.n_receivers], np.int32), np.array([0], np.int32))
        with pytest.raises(P.PahqError):
            gm.eval_edge_list(np.array([0], np.int32), np.array([g.n_upstream(0)], np.int32))
        # a removed set that reaches upstream of a receiver of the list is refused there
        with pytest.raises(P.PahqError):
            gm.eval_edge_list(np.array([g.n_receivers - 1], np.int32), np.array([0], np.int32))
    finally:
        gm.close()


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi", "cfg1_hi"])
def test_layerwise_reference_runs_equal_single_head_runs(name):
    """The reference runs of all heads of a layer as one pass (models with room for H instances) against one pass
    per head (a model whose batch limit is below H): the same reference logits bit for bit, for every head, and the
    same per-edge values -- under both metrics."""
    import paper_2510_23264_amd as P
    import synth
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    H, L = shape.n_heads, shape.n_layers
    g = Graph(L, H, shape.d_mlp > 0)
    ans, dis = synth.make_answers(shape.vocab, B, "uniform", 5)
    one = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=H - 1)       # no room: one reference pass per head
    many = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=max(H, 8))
    try:
        for metric in (P.METRIC_KL, P.METRIC_LOGIT_DIFF):
            for gm in (one, many):
                gm.set_metric(metric, ans, dis)
                gm.clean_cache(clean, corrupt)
            for l in range(L - 1, -1, -1):
                for h in range(H):
                    r = g.headin(l, h, (l + h) % 3)
                    senders = np.arange(g.n_upstream(r), dtype=np.int32)
                    a, b = one.eval_edges(r, senders), many.eval_edges(r, senders)
                    assert np.array_equal(bits(a), bits(b)), (name, metric, l, h)
                    assert np.array_equal(bits(one.get_logits(2)), bits(many.get_logits(2))), (name, metric, l, h)
                    assert one.eval_current(r) == many.eval_current(r)
    finally:
        one.close(); many.close()
