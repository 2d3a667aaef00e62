"""Passes over a pruned graph that leave out dead nodes, against the oracle (which computes every node).

A node is dead once no kept path leads from it to the output: all its outgoing edges are removed, or lead
only to dead nodes.  Every receiver then reads the corrupted run's activation from it (paper, Appendix
"Preliminaries": a removed edge carries the corrupted activation), so the library does not compute it and
lets the stream take its cached corrupted output instead.  The oracle knows nothing of this: it computes
every node of every run.  The removed sets here are built so that single heads, an MLP, a whole attention
layer, a chain (a head whose only kept edge feeds a dead MLP) and all heads of the candidates' own layer
but the investigated one are dead, with random removals on top.
"""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402
from oracle.acdc import MODE_ALL_FP32, MODE_ALL_FP8, MODE_PAHQ   # noqa: E402
from fp32_spread import SpreadModel, kl_with_spread, circuit_kl_with_spread   # noqa: E402
from tolerance import check_kl_cases, tight          # noqa: E402

pytestmark = pytest.mark.gpu


def kill(g, R, sender, from_receiver=0):
    """Removes every edge out of `sender` into receivers >= from_receiver."""
    for r in g.receivers_downstream_of(sender):
        if r >= from_receiver:
            R[r, sender] = True


def scenarios(g, shape, v):
    """Removed sets that touch only receivers at or after receiver v's position (a state of the sweep at v)."""
    L, H, mlp = shape.n_layers, shape.n_heads, shape.d_mlp > 0
    kind, lv, hv, cv = g.receiver_info(v)
    first = v if kind != "headin" else g.headin(lv, 0, 0)      # every receiver of v's layer position may carry removed edges
    rng = np.random.default_rng(100 + v)

    def sprinkle(R, frac):
        for r in range(first, g.n_receivers):
            R[r, : g.n_upstream(r)] |= rng.random(g.n_upstream(r)) < frac
        return R
    out = []
    top = L - 1
    # single heads
    R = g.empty_removed(); kill(g, R, g.head(top, 0), first)
    if lv < top and H > 1: kill(g, R, g.head(top, H - 1), first)
    out.append(("heads", sprinkle(R, 0.2)))
    if mlp:
        R = g.empty_removed(); kill(g, R, g.mlp(top), first)
        if lv + 1 < top: kill(g, R, g.mlp(lv + 1), first)
        out.append(("an MLP", sprinkle(R, 0.3)))
        # a chain: the top MLP is dead, and one head of its layer keeps only its edge into that MLP
        R = g.empty_removed(); kill(g, R, g.mlp(top), first)
        R[g.n_receivers - 1, g.head(top, 0)] = True
        out.append(("a chain", sprinkle(R, 0.1)))
    # a whole attention layer
    R = g.empty_removed()
    for h in range(H): kill(g, R, g.head(top, h), first)
    out.append(("a layer", sprinkle(R, 0.25)))
    if kind == "headin" and H > 1:
        # all heads of the candidates' own layer but the investigated one
        R = g.empty_removed()
        for h in range(H):
            if h != hv: kill(g, R, g.head(lv, h), first)
        out.append(("own layer", sprinkle(R, 0.15)))
    # nearly everything: only the candidates' node (if any) and the embedding still reach the output
    R = g.empty_removed()
    node = g.node_of_receiver(v)
    for s in range(1, g.n_senders):
        if s != node and any(r >= first for r in g.receivers_downstream_of(s)): kill(g, R, s, first)
    out.append(("nearly all", R))
    return out


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi", "cfg1_hi"])
@pytest.mark.parametrize("mode", ["pahq", "all_fp8", "all_fp32"])
def test_states_with_dead_nodes(name, mode):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    om = SpreadModel(shape, w)
    g = om.g
    L, H = shape.n_layers, shape.n_heads
    prec, omode = {"pahq": (P.PAHQ, MODE_PAHQ), "all_fp8": (P.ALL_FP8, MODE_ALL_FP8), "all_fp32": (P.ALL_FP32, MODE_ALL_FP32)}[mode]
    gm = P.Model(shape, w, B, S, precision=prec, max_batch_edges=8)
    try:
        gm.clean_cache(clean, corrupt)
        receivers = [g.headin(0, 0, 1), g.headin(min(1, L - 1), H - 1, 2), g.n_receivers - 1]
        if shape.d_mlp > 0:
            receivers.append(g.mlpin(0))
        cases, labels, got_on, got_off = [], [], [], []
        for v in receivers:
            senders = np.arange(g.n_upstream(v), dtype=np.int32)
            for label, R in scenarios(g, shape, v):
                gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
                gm.set_dead_node_skipping(True)
                on = (gm.eval_current(v), gm.eval_edges(v, senders))
                gm.set_dead_node_skipping(False)
                off = (gm.eval_current(v), gm.eval_edges(v, senders))
                gm.set_dead_node_skipping(True)
                cases.append((v, R, senders)); labels.append((v, label)); got_on.append(on); got_off.append(off)
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        res = kl_with_spread(om, clean, corrupt, omode, cases, seeds=3)
        want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
        sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
        flat = lambda xs: np.concatenate([[c] + list(n) for c, n in xs])
        if mode == "all_fp32":
            # nothing is quantised: binary32 against fp64, with and without the dead nodes
            for what, x in (("skipping", flat(got_on)), ("computing all", flat(got_off))):
                assert (np.abs(x - want) <= 2e-6 + 2e-5 * np.abs(want)).all(), (name, what, float(np.abs(x - want).max()))
        else:
            check_kl_cases(flat(got_on), want, sigma, what=name + " " + mode + " dead nodes skipped")
            check_kl_cases(flat(got_off), want, sigma, what=name + " " + mode + " every node computed")
        # the two device paths against each other: the same sums in a different order
        d = np.abs(flat(got_on) - flat(got_off))
        assert np.median(d / tight(want)) <= 0.05, (name, mode, "median difference between the two paths", float(np.median(d / tight(want))))
        # the scenarios do what they say: where nearly all is removed, candidates from senders whose edges into
        # the candidates' own position are irrelevant still move the metric through the receiver itself
        assert (want > 0).any() and np.isfinite(flat(got_on)).all()
    finally:
        gm.close()


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi"])
def test_circuit_evaluation_with_dead_nodes(name):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    om = SpreadModel(shape, w)
    g = om.g
    L, H = shape.n_layers, shape.n_heads
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=4)
    try:
        gm.clean_cache(clean, corrupt)
        got, got_off, want, sigma = [], [], [], []
        for label, R in scenarios(g, shape, 0):                  # receiver 0: any receiver may carry removed edges
            kept = (~g.removed_to_flat(R)).astype(np.uint8)
            for flags in (np.zeros((L, H), np.uint8), np.ones((L, H), np.uint8)):
                pi = frozenset((l, h) for l in range(L) for h in range(H) if flags[l, h])
                gm.set_dead_node_skipping(True)
                kl, logits = gm.eval_circuit(kept=kept, f32_heads=flags, want_logits=True)
                gm.set_dead_node_skipping(False)
                kl_off = gm.eval_circuit(kept=kept, f32_heads=flags)
                gm.set_dead_node_skipping(True)
                o_kl, o_logits, s = circuit_kl_with_spread(om, clean, corrupt, pi, R, seeds=3)
                got.append(kl); got_off.append(kl_off); want.append(o_kl); sigma.append(s)
                assert np.abs(logits - o_logits).max() <= 0.1 * np.abs(o_logits).max(), (name, label)
        check_kl_cases(got, want, sigma, what=name + " circuit, dead nodes skipped")
        check_kl_cases(got_off, want, sigma, what=name + " circuit, every node computed")
    finally:
        gm.close()
