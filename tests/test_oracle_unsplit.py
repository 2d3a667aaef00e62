"""Pins of the coarser graph (one input per head, read by its query, key and value projections alike):
its ids and edge count by their definitions, and its forward and edge scores against the split graph
(whose routing is pinned on its own) with the three inputs of a head treated alike."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import synth                                           # noqa: E402
from oracle.graph import Graph                         # noqa: E402
from oracle.model import Model                         # noqa: E402
from oracle.acdc import Acdc, MODE_PAHQ, MODE_ALL_FP8  # noqa: E402
from loop_forward import loop_forward                  # noqa: E402
from test_oracle_model import tiny, TINY_GELU, TINY_LLAMA, TINY_ATTN, _names, _rel     # noqa: E402


def test_ids_and_edge_count():
    s = synth.make_shape("cfg3")
    g = Graph(s.n_layers, s.n_heads, True, split_qkv=False)
    assert g.n_edges() == 11611                        # GPT-2-small shape: a third of the head-input edges of the split graph
    g3 = Graph(s.n_layers, s.n_heads, True)
    head_edges3 = sum(g3.n_upstream(g3.headin(l, h, c)) for l in range(12) for h in range(12) for c in range(3))
    assert g3.n_edges() - g.n_edges() == head_edges3 * 2 // 3
    for L, H, mlp in ((1, 1, False), (2, 3, True), (3, 2, False), (4, 4, True)):
        g = Graph(L, H, mlp, split_qkv=False)
        seen = set()
        for r in range(g.n_receivers):
            kind, l, h, c = g.receiver_info(r)
            rid = g.OUT if kind == "out" else (g.mlpin(l) if kind == "mlpin" else g.headin(l, h))
            assert rid == r and c == -1
            seen.add(rid)
            if kind == "headin":
                assert g.headin(l, h, 0) == g.headin(l, h, 2) == r and g.node_of_receiver(r) == g.head(l, h)
            # upstream by the definition: the embedding, every node of an earlier layer, and for an MLP input the heads of its own
            n = 1 + sum(1 for s in range(1, g.n_senders)
                        if g.sender_info(s)[1] < l or (kind == "mlpin" and g.sender_info(s) [0] == "head" and g.sender_info(s)[1] == l))
            assert g.n_upstream(r) == (g.n_senders if kind == "out" else n)
        assert len(seen) == g.n_receivers == L * (H + (1 if mlp else 0)) + 1


def to_split(g1, g3, R1):
    """The removed set of the split graph that treats the three inputs of every head like the one input."""
    R3 = g3.empty_removed()
    for r in range(g1.n_receivers):
        kind, l, h, _ = g1.receiver_info(r)
        targets = [g3.OUT] if kind == "out" else ([g3.mlpin(l)] if kind == "mlpin" else [g3.headin(l, h, c) for c in range(3)])
        for t in targets:
            R3[t, : g1.n_upstream(r)] = R1[r, : g1.n_upstream(r)]
    return R3


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
def test_forward_equals_the_split_graph_with_tied_inputs(shape):
    m3, w, clean, corrupt = tiny(shape, B=2)
    m1 = Model(shape, w, split_qkv=False)
    g1, g3 = m1.g, m3.g
    rng = np.random.default_rng(5)
    snd, rcv3 = _names(g3)
    for pi in (frozenset(), frozenset([(1, 0)])):
        C, _ = m3.forward(corrupt, pi)
        C1, _ = m1.forward(corrupt, pi)
        assert np.array_equal(C, C1)
        for frac in (0.0, 0.3, 0.8):
            R1 = g1.empty_removed()
            for r in range(g1.n_receivers):
                R1[r, : g1.n_upstream(r)] = rng.random(g1.n_upstream(r)) < frac
            R3 = to_split(g1, g3, R1)
            o1, l1 = m1.forward(clean, pi, removed=R1, C=C)
            o3, l3 = m3.forward(clean, pi, removed=R3, C=C)
            assert np.array_equal(l1, l3) and np.array_equal(o1, o3), (sorted(pi), frac)
        # ... and against the independent loop forward, the same edge removed from q, k and v
        R1 = g1.empty_removed()
        for r in range(g1.n_receivers):
            R1[r, : g1.n_upstream(r)] = rng.random(g1.n_upstream(r)) < 0.4
        R3 = to_split(g1, g3, R1)
        rem = frozenset((snd[s], rcv3[r]) for r in range(g3.n_receivers) for s in range(g3.n_upstream(r)) if R3[r, s])
        other = {snd[s]: C[s].reshape(-1, shape.d_model) for s in range(g3.n_senders)}
        _, lg = m1.forward(clean, pi, removed=R1, C=C)
        _, l_lg = loop_forward(shape, w, clean, pi=pi, removed=rem, other=other)
        assert _rel(lg, l_lg) < 1e-12


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_ATTN])
def test_edge_scores_and_sweep_on_the_coarser_graph(shape):
    m3, w, clean, corrupt = tiny(shape, B=2)
    m1 = Model(shape, w, split_qkv=False)
    for mode in (MODE_PAHQ, MODE_ALL_FP8):
        a = Acdc(m1, clean, corrupt, mode)
        g = a.g
        R = g.empty_removed()
        for r in range(g.n_receivers):
            for u in range(g.n_upstream(r)):
                assert abs(a.kl_edge(r, u, removed=R) - a.kl_edge(r, u, removed=R, brute=True)) < 1e-12, (mode, r, u)
        kls = sorted(a.kl_edge(r, u) for r in range(g.n_receivers) for u in range(g.n_upstream(r)))
        tau = kls[len(kls) // 2]
        rem_fast, tr_fast = a.sweep(tau)
        rem_brute, tr_brute = Acdc(m1, clean, corrupt, mode).sweep(tau, brute=True)
        assert np.array_equal(rem_fast, rem_brute) and len(tr_fast) == len(tr_brute)
        assert 0 < rem_fast.sum() < g.n_edges()
        # the fp32 head of a candidate is the head its edge feeds
        assert a.pi_of(g.headin(1, 0)) == (frozenset([(1, 0)]) if mode == MODE_PAHQ else frozenset())
