"""The coarser graph (pahq_config.split_qkv = 0: a head has one input that its query, key and value projections all
read) on the device against the oracle on the same graph: per-edge values and states under per-head mixed precision
and all-8-bit, sweeps decision by decision, exact zero for identical prompts, circuit evaluation, edge lists."""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402
from fp32_spread import kl_with_spread, circuit_kl_with_spread     # noqa: E402
from tolerance import check_kl_cases                # noqa: E402
from test_gpu_parity import Pair, compare_sweep, random_removed     # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["cfg1_hi", "mid_hi", "midllama_hi"])
@pytest.mark.parametrize("precision", [2, 1, 0])
def test_coarser_graph(name, precision):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    pr = Pair(shape, w, clean, corrupt, precision=precision, split_qkv=False, max_batch=8)
    try:
        g, gm = pr.g, pr.gm
        L, H = shape.n_layers, shape.n_heads
        assert gm.n_edges == g.n_edges() and g.n_receivers == L * (H + (1 if shape.d_mlp else 0)) + 1
        receivers = [g.OUT, g.headin(L - 1, H - 1), g.headin(0, 0), g.headin(min(1, L - 1), 0)] + ([g.mlpin(L - 1)] if shape.d_mlp else [])
        cases, got = [], []
        for i, r in enumerate(receivers):
            R = g.empty_removed() if i % 2 == 0 else random_removed(g, 0.4, 41 + i, from_receiver=r)
            senders = np.arange(g.n_upstream(r), dtype=np.int32)
            gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
            vals = gm.eval_edges(r, senders)
            # the list form gives the same bits
            assert np.array_equal(gm.eval_edge_list(np.full(len(senders), r, np.int32), senders).view(np.uint32), vals.view(np.uint32))
            got.append(np.concatenate([[gm.eval_current(r)], vals]))
            cases.append((r, R, senders))
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        res = kl_with_spread(pr.om, clean, corrupt, pr.mode, cases, seeds=4)
        want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
        sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
        worst = check_kl_cases(np.concatenate(got), want, sigma, what=name + " coarser graph")
        print(name, "precision", precision, "coarser graph: median KL %.3g, worst |d| / bound %.3f" % (np.median(want), worst))
        # a whole list over every receiver equals the per-receiver calls
        rr = np.concatenate([np.full(g.n_upstream(r), r, np.int32) for r in range(g.n_receivers)])
        ss = np.concatenate([np.arange(g.n_upstream(r), dtype=np.int32) for r in range(g.n_receivers)])
        per = np.concatenate([gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) for r in range(g.n_receivers)])
        assert np.array_equal(gm.eval_edge_list(rr, ss).view(np.uint32), per.view(np.uint32))
        # sweeps
        taus = {"cfg1_hi": (0.05, 0.3), "mid_hi": (0.01,), "midllama_hi": (0.03,)}[name]
        outcomes = [compare_sweep(pr, tau)[0] for tau in taus]
        assert "equal" in outcomes, outcomes
        # a pruned graph under a set of fp32 heads
        if precision == 2:
            R = random_removed(g, 0.5, 9)
            flags = np.zeros((L, H), np.uint8); flags[L - 1, 0] = flags[0, H - 1] = 1
            pi = frozenset((l, h) for l in range(L) for h in range(H) if flags[l, h])
            kl = gm.eval_circuit(kept=(~g.removed_to_flat(R)).astype(np.uint8), f32_heads=flags)
            o_kl, _, s = circuit_kl_with_spread(pr.om, clean, corrupt, pi, R, seeds=3)
            check_kl_cases([kl], [o_kl], [s], what=name + " coarser graph, circuit", median_rule=False)
    finally:
        pr.close()
    # identical prompts: exactly zero (every node computed)
    gm = P.Model(shape, w, clean.shape[0], clean.shape[1], precision=precision, max_batch_edges=8, split_qkv=False)
    try:
        gm.clean_cache(clean, clean.copy())
        gm.set_dead_node_skipping(False)
        for r in (g.OUT, g.headin(L - 1, 0), g.headin(0, H - 1)):
            gm.set_removed(g.removed_to_flat(random_removed(g, 0.5, 3, from_receiver=r)).astype(np.uint8))
            assert (gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) == 0.0).all() and gm.eval_current(r) == 0.0
    finally:
        gm.close()


def test_options_compose():
    """The coarser graph, the 4-bit grid for the heads and bfloat16 for everything else, in one model, on a pruned
    state with dead nodes: against the oracle with the same three options."""
    shape, w, clean, corrupt = workloads.make("mid_hi")
    pr = Pair(shape, w, clean, corrupt, split_qkv=False, low_bits=4, nonattn_bf16=True, max_batch=8)
    try:
        g, gm = pr.g, pr.gm
        L, H = shape.n_layers, shape.n_heads
        cases, got = [], []
        for i, r in enumerate((g.OUT, g.headin(L - 1, 1), g.mlpin(0), g.headin(0, 0))):
            R = random_removed(g, 0.5, 61 + i, from_receiver=r)
            for s in (g.head(L - 1, 0), g.mlp(L - 1)):                   # two dead nodes
                for t in g.receivers_downstream_of(s):
                    if t >= r:
                        R[t, s] = True
            senders = np.arange(g.n_upstream(r), dtype=np.int32)
            gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
            got.append(np.concatenate([[gm.eval_current(r)], gm.eval_edges(r, senders)]))
            cases.append((r, R, senders))
        res = kl_with_spread(pr.om, clean, corrupt, pr.mode, cases, seeds=3)
        want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
        sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
        check_kl_cases(np.concatenate(got), want, sigma, what="options together")
        assert np.median(want) > 1e-3
    finally:
        pr.close()
