"""Pins for the oracle's forward, graph, scoring and sweep (CPU only)."""
import json
import math
import os
import numpy as np
import pytest

import synth
from synth import ModelShape
from oracle import e4m3
from oracle.graph import Graph
from oracle.model import (Model, ALL, NONE, layer_norm, rms_norm, gelu_tanh, silu, log_softmax,
                          kl_to_reference)
from oracle.acdc import Acdc, MODE_ALL_FP32, MODE_ALL_FP8, MODE_PAHQ
from plain_forward import plain_forward

FACTS = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))

TINY_GELU = ModelShape(n_layers=2, n_heads=2, d_head=8, d_model=16, d_mlp=32, vocab=40, n_ctx=6)
TINY_LLAMA = ModelShape(n_layers=2, n_heads=2, d_head=8, d_model=16, d_mlp=24, vocab=40, n_ctx=6,
                        norm=1, act=2, pos=1, norm_eps=1e-6)
TINY_ATTN = ModelShape(n_layers=2, n_heads=3, d_head=4, d_model=12, d_mlp=0, vocab=30, n_ctx=5, act=0)


def tiny(shape, seed=3, B=3, S=None, k=2):
    S = S or shape.n_ctx
    w = synth.make_weights(shape, seed, std=0.3, affine_std=0.2)
    clean, corrupt = synth.make_tokens(shape.vocab, B, S, "uniform", k, False, seed)
    return Model(shape, w), w, clean, corrupt


# ---------------------------------------------------------------- graph
def test_edge_counts():
    expect = {"cfg1": 81, "cfg2": 1519, "cfg3": 32491, "cfg4": 231877, "cfg5": 1592881}
    for name, n in expect.items():
        s = synth.make_shape(name)
        g = Graph(s.n_layers, s.n_heads, s.d_mlp > 0)
        assert g.n_edges() == n, name
    # the paper's "about 35,000 edges" for GPT-2 small picks the split-QKV graph
    f = FACTS["gpt2_small_start_edges_approx"]
    assert abs(32491 - f["value"]) <= f["rel_tol"] * f["value"]
    # brute-force count from the definition of "upstream" on a small graph
    g = Graph(3, 2, True)
    n = 0
    for r in range(g.n_receivers):
        kind, l, _, _ = g.receiver_info(r)
        for s in range(g.n_senders):
            sk, sl, _ = g.sender_info(s)
            up = (sk == "embed" or kind == "out"
                  or (kind == "headin" and sl < l)
                  or (kind == "mlpin" and (sl < l or (sl == l and sk == "head"))))
            assert up == (s < g.n_upstream(r))
            n += up
    assert n == g.n_edges()
    assert g.receiver_info(g.headin(2, 1, 2)) == ("headin", 2, 1, 2)
    assert g.node_of_receiver(g.mlpin(1)) == g.mlp(1) and g.node_of_receiver(g.OUT) == -1
    flat = np.arange(g.n_edges()) % 3 == 0
    assert (g.removed_to_flat(g.flat_to_removed(flat)) == flat).all()


# ---------------------------------------------------------------- pieces
def test_norms_activations_softmax_kl():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 32)) * 3 + 1
    y = layer_norm(x, np.ones(32), np.zeros(32), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-14) and np.allclose((y * y).mean(-1), 1, atol=1e-12)
    y = rms_norm(x, np.ones(32), 0.0)
    assert np.allclose((y * y).mean(-1), 1, atol=1e-12)
    t = np.linspace(-6, 6, 41)
    ref = np.array([0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3))) for v in t])
    assert np.allclose(gelu_tanh(t), ref, atol=1e-15)
    erf_form = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in t])
    assert np.abs(gelu_tanh(t) - erf_form).max() < 5e-3          # tanh form approximates the erf form
    assert np.allclose(silu(t), [v / (1 + math.exp(-v)) for v in t], atol=1e-15)
    lp = log_softmax(x)
    assert np.allclose(np.exp(lp).sum(-1), 1, atol=1e-14)
    # KL: zero iff equal, invariant to a logit shift, non-negative, two-token closed form
    assert kl_to_reference(lp, x) == 0.0
    assert abs(kl_to_reference(lp, x + 7.5)) < 1e-14
    assert kl_to_reference(lp, rng.standard_normal((5, 32))) > 0
    p, q = 0.3, 0.6
    lg_p = np.log(np.array([[p, 1 - p]])); lg_q = np.log(np.array([[q, 1 - q]]))
    closed = p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q))
    assert abs(kl_to_reference(log_softmax(lg_p), lg_q) - closed) < 1e-15


def test_rope_is_a_relative_rotation():
    m, _, _, _ = tiny(TINY_LLAMA)
    rng = np.random.default_rng(1)
    B, S, dh = 1, 6, TINY_LLAMA.d_head
    q, k = rng.standard_normal((S, dh)), rng.standard_normal((S, dh))
    rq, rk = m._rope(q, B, S), m._rope(k, B, S)
    assert np.allclose((rq * rq).sum(-1), (q * q).sum(-1))          # a rotation keeps the norm
    assert np.allclose(rq[0], q[0])                                  # position 0 is the identity
    # same vectors placed at (i, j) and (i+2, j+2) give the same score
    q2 = np.tile(q[1], (S, 1)); k2 = np.tile(k[4], (S, 1))
    r1, r2 = m._rope(q2, B, S), m._rope(k2, B, S)
    assert abs(r1[3] @ r2[1] - r1[5] @ r2[3]) < 1e-12
    assert abs(r1[3] @ r2[1] - r1[3] @ r2[2]) > 1e-6


# ---------------------------------------------------------------- forward
@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
def test_all_fp32_equals_plain_forward(shape):
    m, w, clean, _ = tiny(shape)
    _, lg = m.forward(clean, ALL)
    ref = plain_forward(shape, w, clean)
    assert np.abs(lg - ref).max() < 1e-11 * max(1.0, np.abs(ref).max())


def test_cfg1_all_fp32_equals_plain_forward():
    shape, w, clean, _, _ = synth.make_workload("cfg1", affine_std=0.1)
    _, lg = Model(shape, w).forward(clean, ALL)
    assert np.abs(lg - plain_forward(shape, w, clean)).max() < 1e-12


def test_fp8_gemm_is_the_quantised_product():
    """One linear map of the model, checked against the definition spelled out
    element by element with Python floats."""
    m, w, clean, _ = tiny(TINY_GELU)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 16))
    y = m._linear(x, "W_Q", (1, 0), True, w["b_Q"][1, 0])
    t = e4m3.decode_table()
    wc, ws = e4m3.quantize_groups(w["W_Q"][1, 0], axis=None)
    assert ws == m.qs["W_Q"][1, 0] and (wc == m.qc["W_Q"][1, 0]).all()
    xc, xs = e4m3.quantize_rows(x.astype(np.float32))
    for r in range(4):
        for j in range(8):
            acc = sum(float(t[xc[r, kk]]) * float(t[wc[kk, j]]) for kk in range(16))
            assert abs(acc * float(xs[r]) * float(ws) + float(w["b_Q"][1, 0, j]) - y[r, j]) < 1e-13
    # weight codes of a layer matrix use one scale for the whole matrix
    c_in, s_in = e4m3.quantize_groups(w["W_in"][1], axis=None)
    assert s_in == m.qs["W_in"][1] and (c_in == m.qc["W_in"][1]).all()
    # quantised forward differs from the plain one, but only by quantisation noise
    _, lq = m.forward(clean, NONE)
    _, lf = m.forward(clean, ALL)
    rel = np.abs(lq - lf).max() / np.abs(lf).max()
    assert 1e-6 < rel < 0.2
    # a head in the precision set changes that head and nothing upstream of it
    o_none, _ = m.forward(clean, NONE)
    o_pi, _ = m.forward(clean, frozenset([(1, 0)]))
    g = m.g
    assert (o_none[: g.head(1, 0)] == o_pi[: g.head(1, 0)]).all()
    assert np.abs(o_none[g.head(1, 0)] - o_pi[g.head(1, 0)]).max() > 0
    assert (o_none[g.head(1, 1)] == o_pi[g.head(1, 1)]).all()


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
@pytest.mark.parametrize("mode", [MODE_PAHQ, MODE_ALL_FP8, MODE_ALL_FP32])
def test_patching_properties(shape, mode):
    m, w, clean, corrupt = tiny(shape)
    g = m.g
    rng = np.random.default_rng(5)
    rand_R = g.flat_to_removed(rng.random(g.n_edges()) < 0.4)

    # P1: corrupt == clean  =>  every patched run reproduces the clean logits, KL = 0 exactly
    a0 = Acdc(m, clean, clean, mode)
    for v in (g.OUT, g.headin(1, 1, 1), g.headin(0, 0, 2)) + ((g.mlpin(0),) if shape.d_mlp else ()):
        assert a0.kl_fast(v, rand_R) == 0.0
        assert a0.kl_brute(v, rand_R) == 0.0

    a = Acdc(m, clean, corrupt, mode)
    # full ablation: every edge removed  =>  logits of the corrupted run; KL = KL(clean || corrupt)
    full = g.flat_to_removed(np.ones(g.n_edges(), bool))
    for v in (g.OUT, g.headin(1, 0, 0)):
        pi = a.pi_of(v)
        C, lg_corrupt = m.forward(corrupt, pi)
        _, lg = m.forward(clean, pi, removed=full, C=C)
        assert np.abs(lg - lg_corrupt).max() < 1e-12
        _, ref = m.forward(clean, pi)
        assert abs(a.kl_brute(v, full) - kl_to_reference(log_softmax(ref), lg_corrupt)) < 1e-13
    # R = empty  =>  KL = 0 exactly
    assert a.kl_fast(g.headin(1, 0, 1), g.empty_removed()) == 0.0

    # dead node: a node without kept out-edges has in-edges of no effect
    dead = g.head(0, 1)
    R = rand_R.copy()
    for r in g.receivers_downstream_of(dead):
        R[r, dead] = True
    v = g.headin(0, 1, 2)
    R[v, :] = False
    k0 = a.kl_fast(v, R)
    R2 = R.copy(); R2[v, 0] = True
    assert a.kl_fast(v, R2) == k0

    # OUT receiver closed form: logits = unembed(norm(resid - (clean_u - corrupt_u)))
    pi = a.pi_of(g.OUT)
    oc, _ = m.forward(clean, pi)
    ox, _ = m.forward(corrupt, pi)
    T, d = clean.size, shape.d_model
    B, S = clean.shape
    for u in (0, g.n_senders - 1, g.head(0, 1)):
        resid = oc.sum(0).reshape(T, d) + m.bias_prefix(g.OUT)
        x = resid - (oc[u] - ox[u]).reshape(T, d)
        xn = m.norm(x.reshape(B, S, d)[:, -1], "lnf")
        lg = m._linear(xn, "W_U", (), pi != ALL, w["b_U"])
        _, ref = m.forward(clean, pi)
        expect = kl_to_reference(log_softmax(ref), lg)
        got = a.kl_edge(g.OUT, u)
        assert abs(got - expect) <= 1e-12 * max(1.0, abs(expect))
        # the embedding is identical at the (never resampled) last position: no effect on OUT
        assert (got == 0.0) if u == 0 else (got > 0)


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA])
def test_brute_force_equals_fast_path_every_edge(shape):
    m, w, clean, corrupt = tiny(shape)
    g = m.g
    a = Acdc(m, clean, corrupt, MODE_PAHQ)
    rng = np.random.default_rng(7)
    for r in range(g.n_receivers):
        R = g.empty_removed()
        # removed sets may only touch receivers >= r (the state the sweep is in when it visits r)
        for r2 in range(r, g.n_receivers):
            R[r2, : g.n_upstream(r2)] = rng.random(g.n_upstream(r2)) < 0.5
        for u in range(g.n_upstream(r)):
            R2 = R.copy(); R2[r, u] = True
            kb, kf = a.kl_brute(r, R2), a.kl_fast(r, R2)
            assert abs(kb - kf) <= 1e-13 * max(1.0, abs(kb)), (r, u)


def test_cfg1_brute_equals_fast_all_81_edges_and_sweep():
    shape, w, clean, corrupt, spec = synth.make_workload("cfg1")
    m = Model(shape, w)
    a = Acdc(m, clean, corrupt, MODE_PAHQ)
    g = m.g
    assert g.n_edges() == 81
    for r in range(g.n_receivers):
        for u in range(g.n_upstream(r)):
            kb, kf = a.kl_edge(r, u, brute=True), a.kl_edge(r, u)
            assert abs(kb - kf) <= 1e-14 + 1e-12 * abs(kb)
    for tau in (spec["taus"][0], 2e-5, 2e-6):
        rf, tf = a.sweep(tau)
        rb, tb = Acdc(m, clean, corrupt, MODE_PAHQ).sweep(tau, brute=True)
        assert (rf == rb).all() and len(tf) == len(tb)
        assert all(x[:2] == y[:2] and x[4] == y[4] and abs(x[2] - y[2]) < 1e-13 for x, y in zip(tf, tb))
    # the small thresholds give non-trivial circuits (some edges kept, some removed)
    kept = (~g.removed_to_flat(rf)).sum()
    assert 0 < kept < 81


def test_sweep_semantics_on_tiny_model():
    m, w, clean, corrupt = tiny(TINY_GELU, B=4)
    g = m.g
    a = Acdc(m, clean, corrupt, MODE_PAHQ)
    base = a.kl_fast(g.OUT, g.empty_removed())
    assert base == 0.0
    removed, trace = a.sweep(1e-3)
    flat = g.removed_to_flat(removed)
    # every edge is either evaluated once or skipped because its node was dead at that time
    evaluated = {(v, u) for v, u, *_ in trace}
    assert len(evaluated) == len(trace)
    # receivers are visited in descending order, senders in descending order
    order = [(v, u) for v, u, *_ in trace]
    assert order == sorted(order, reverse=True)
    # decisions follow the rule, and kl_cur chains through accepted removals
    for i, (v, u, kn, kc, rm) in enumerate(trace):
        assert rm == ((kn - kc) < 1e-3)
    # an edge that was never evaluated belongs to a dead node and is removed
    for r in range(g.n_receivers):
        for u in range(g.n_upstream(r)):
            if (r, u) not in evaluated:
                assert removed[r, u]
                assert not a.node_is_live(r, removed)
    # tau = +inf removes everything it evaluates; tau = -inf keeps everything
    r_all, t_all = a.sweep(float("inf"))
    assert g.removed_to_flat(r_all).all() and len(t_all) == g.n_upstream(g.OUT)
    r_none, t_none = a.sweep(-float("inf"))
    assert not g.removed_to_flat(r_none).any() and len(t_none) == g.n_edges()
    assert all(abs(kc) == 0.0 for *_, kc, _ in t_none)


def test_interrupted_sweep_continues_from_its_removed_set():
    """The pass decides receiver by receiver, every decision given all earlier ones (Appendix "Preliminaries", pruning
    rule): cut anywhere between two receivers, the removed set reached so far is the whole state."""
    m, w, clean, corrupt = tiny(TINY_GELU, B=4)
    g = m.g
    a = Acdc(m, clean, corrupt, MODE_PAHQ)
    for tau in (1e-3, 1e-5):
        full, t_full = a.sweep(tau)
        for cut in (g.n_receivers - 1, g.n_receivers // 2, 1):
            upper, t1 = a.sweep(tau, receivers=range(cut, g.n_receivers))
            both, t2 = a.sweep(tau, receivers=range(0, cut), start=upper)
            assert (both == full).all() and t1 + t2 == t_full, (tau, cut)


def test_sequence_order_does_not_matter():
    m, w, clean, corrupt = tiny(TINY_LLAMA, B=4)
    g = m.g
    perm = np.array([2, 0, 3, 1])
    v = g.headin(1, 0, 0)
    R = g.empty_removed(); R[v, 1] = True; R[g.OUT, 3] = True
    a, b = Acdc(m, clean, corrupt), Acdc(m, clean[perm], corrupt[perm])
    la, lb = a.logits_fast(v, R), b.logits_fast(v, R)
    assert (la[perm] == lb).all()


def test_pahq_keeps_what_rtn_loses():
    """The mechanism the paper describes: with everything in 8 bits a small
    activation difference can vanish in the receiver's quantised input; the fp32
    receiver head sees it.  Checked on the logits' sensitivity to one edge."""
    m, w, clean, corrupt = tiny(TINY_GELU, B=4)
    g = m.g
    v = g.headin(1, 0, 1)          # a key input: earlier positions reach the last position's logits
    kl32 = Acdc(m, clean, corrupt, MODE_ALL_FP32).kl_edge(v, 0)
    klp = Acdc(m, clean, corrupt, MODE_PAHQ).kl_edge(v, 0)
    klq = Acdc(m, clean, corrupt, MODE_ALL_FP8).kl_edge(v, 0)
    assert kl32 > 0 and klp > 0
    assert klp != klq


# ---------------------------------------------------------------- pins by an independent loop forward
from loop_forward import loop_forward, SITES


def _names(g):
    """id -> tuple name of every sender and receiver (the id formulas are pinned by test_edge_counts)."""
    snd = {}
    for s in range(g.n_senders):
        kind, l, h = g.sender_info(s)
        snd[s] = ("embed",) if kind == "embed" else (("head", l, h) if kind == "head" else ("mlp", l))
    rcv = {}
    for r in range(g.n_receivers):
        kind, l, h, c = g.receiver_info(r)
        rcv[r] = ("out",) if kind == "out" else (("mlpin", l) if kind == "mlpin" else ("qkv"[c], l, h))
    return snd, rcv


def _rel(a, b):
    return np.abs(a - b).max() / max(1.0, np.abs(b).max())


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
def test_quantiser_placement_against_loop_forward(shape):
    """Every operand the method quantises, and no other, is quantised: the oracle's forward under
    several precision sets equals a forward written out with explicit loops; leaving out any single
    quantiser in that forward is seen (so a quantiser missing from, or added to, the oracle would be)."""
    m, w, clean, _ = tiny(shape, B=2)
    snd, _ = _names(m.g)
    sets = [frozenset(), frozenset([(1, 0)]), frozenset([(0, 1)]), frozenset([(0, 0), (1, 1)])]
    for pi in sets:
        outs, lg = m.forward(clean, pi)
        l_out, l_lg = loop_forward(shape, w, clean, pi=pi)
        assert _rel(lg, l_lg) < 1e-12, sorted(pi)
        for s, nm in snd.items():
            assert _rel(outs[s].reshape(l_out[nm].shape), l_out[nm]) < 1e-12, (sorted(pi), nm)
    outs, lg = m.forward(clean, ALL)
    _, l_lg = loop_forward(shape, w, clean, quantise=False)
    assert _rel(lg, l_lg) < 1e-12
    # sensitivity: one quantiser left out of the loop forward is a visible difference
    pi = frozenset([(1, 0)])
    _, lg = m.forward(clean, pi)
    for site in SITES:
        if shape.d_mlp == 0 and site in ("act:in", "w:in", "w:gate", "act:out", "w:out"):
            continue
        if shape.act != 2 and site == "w:gate":
            continue
        _, l_lg = loop_forward(shape, w, clean, pi=pi, drop=site)
        assert _rel(lg, l_lg) > 1e-7, site
    # ... and so is a head of the precision set that is quantised after all, or one too many in fp32
    _, l_lg = loop_forward(shape, w, clean, pi=frozenset())
    assert _rel(lg, l_lg) > 1e-7
    _, l_lg = loop_forward(shape, w, clean, pi=frozenset([(1, 0), (1, 1)]))
    assert _rel(lg, l_lg) > 1e-7


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
def test_patch_routing_against_loop_forward(shape):
    """A removed edge replaces one sender's output at one receiver -- one channel of one head, one MLP
    input, or the unembedding input -- and nowhere else: random removed sets, explicit per-receiver sums."""
    m, w, clean, corrupt = tiny(shape, B=2)
    g = m.g
    snd, rcv = _names(g)
    rng = np.random.default_rng(11)
    for pi in (frozenset(), frozenset([(1, 1)])):
        C, _ = m.forward(corrupt, pi)
        other = {snd[s]: C[s].reshape(clean.size, shape.d_model) for s in snd}
        for frac in (0.15, 0.6):
            R = g.flat_to_removed(rng.random(g.n_edges()) < frac)
            rem = {(snd[s], rcv[r]) for r in range(g.n_receivers) for s in range(g.n_upstream(r)) if R[r, s]}
            outs, lg = m.forward(clean, pi, removed=R, C=C)
            l_out, l_lg = loop_forward(shape, w, clean, pi=pi, removed=rem, other=other)
            assert _rel(lg, l_lg) < 1e-12
            for s, nm in snd.items():
                assert _rel(outs[s].reshape(l_out[nm].shape), l_out[nm]) < 1e-12, nm
            # sensitivity: the same edges routed into another channel of the same head give something else
            swap = {"q": "k", "k": "v", "v": "q"}
            rem2 = {(s_, (swap[r_[0]],) + r_[1:] if r_[0] in swap else r_) for s_, r_ in rem}
            if rem2 != rem:
                _, l_lg2 = loop_forward(shape, w, clean, pi=pi, removed=rem2, other=other)
                assert _rel(lg, l_lg2) > 1e-7
    # one edge at a time: the patched run differs from the clean run only downstream of the receiver's node
    C, _ = m.forward(corrupt, frozenset())
    base, _ = m.forward(clean, frozenset())
    v = g.headin(1, 0, 2)
    R = g.empty_removed(); R[v, g.head(0, 1)] = True
    outs, _ = m.forward(clean, frozenset(), removed=R, C=C)
    changed = [s for s in range(g.n_senders) if not (outs[s] == base[s]).all()]
    assert changed and changed[0] == g.head(1, 0) and g.head(1, 1) not in changed


# ---------------------------------------------------------------- logit-difference task metric
from oracle.acdc import METRIC_LOGIT_DIFF, logit_diff_drop


def test_logit_difference_metric():
    """Paper, Appendix "Task Metrics": the logit of the correct answer minus that of a distractor.  As a
    loss relative to the clean reference it is 0 for the unpruned graph, the drop ld(clean) - ld(corrupt) for
    the fully ablated one, unchanged by a per-sequence shift of the logits, and written out per sequence it is
    what the function returns."""
    m, w, clean, corrupt = tiny(TINY_GELU, B=4)
    g = m.g
    ans, dis = synth.make_answers(TINY_GELU.vocab, 4, "uniform", 9)
    assert (ans != dis).all()
    rng = np.random.default_rng(1)
    ref, lg = rng.standard_normal((4, 40)), rng.standard_normal((4, 40))
    by_hand = np.mean([(ref[b, ans[b]] - ref[b, dis[b]]) - (lg[b, ans[b]] - lg[b, dis[b]]) for b in range(4)])
    assert abs(logit_diff_drop(ref, lg, ans, dis) - by_hand) < 1e-15
    assert logit_diff_drop(ref, ref, ans, dis) == 0.0
    assert abs(logit_diff_drop(ref, lg + rng.standard_normal((4, 1)), ans, dis) - by_hand) < 1e-14
    a = Acdc(m, clean, corrupt, MODE_PAHQ, metric=METRIC_LOGIT_DIFF, answer=ans, distractor=dis)
    v = g.headin(1, 0, 1)
    assert a.kl_fast(v, g.empty_removed()) == 0.0
    full = g.flat_to_removed(np.ones(g.n_edges(), bool))
    pi = a.pi_of(v)
    _, lc = m.forward(clean, pi)
    _, lx = m.forward(corrupt, pi)
    b = np.arange(4)
    drop = ((lc[b, ans] - lc[b, dis]) - (lx[b, ans] - lx[b, dis])).mean()
    assert abs(a.kl_brute(v, full) - drop) < 1e-12
    # brute force (three forwards) = cached fast path, and a clean patch scores exactly 0
    R = g.flat_to_removed(rng.random(g.n_edges()) < 0.4)
    for r in (g.OUT, g.mlpin(1), v):
        Rr = R.copy(); Rr[:r] = False
        for u in (0, g.n_upstream(r) - 1):
            assert abs(a.kl_edge(r, u, removed=Rr) - a.kl_edge(r, u, removed=Rr, brute=True)) < 1e-13
    a0 = Acdc(m, clean, clean, MODE_PAHQ, metric=METRIC_LOGIT_DIFF, answer=ans, distractor=dis)
    assert a0.kl_fast(v, R * 0 + (np.arange(g.n_receivers)[:, None] >= v) * R) == 0.0
    # the sweep runs on it with the same rule
    removed, trace = a.sweep(1e-3)
    assert all(rm == ((kn - kc) < 1e-3) for _, _, kn, kc, rm in trace)


def test_sender_side_precision_policy():
    """Eq. P_t as printed (fp32 for the source of the evaluated edge): the cached evaluation from the sender's layer
    equals three-plus-one full forwards under that set; a clean patch scores 0; with everything in fp32 the two
    policies are the same procedure; under mixed precision they are different numbers."""
    m, w, clean, corrupt = tiny(TINY_GELU, B=3)
    g = m.g
    a = Acdc(m, clean, corrupt, MODE_PAHQ)
    rng = np.random.default_rng(4)
    v = g.headin(1, 1, 2)
    R = g.empty_removed(); R[v:, :] = g.flat_to_removed(rng.random(g.n_edges()) < 0.4)[v:, :]
    for u in (g.head(0, 1), g.mlp(0), 0):
        cur, new = a.pair_sender_policy(v, u, R)
        pi = a.pi_of_sender(u)
        assert pi == (frozenset([(0, 1)]) if u == g.head(0, 1) else frozenset())
        C, _ = m.forward(corrupt, pi)
        _, ref = m.forward(clean, pi)
        _, lc = m.forward(clean, pi, removed=R, C=C)
        R2 = R.copy(); R2[v, u] = True
        _, ln = m.forward(clean, pi, removed=R2, C=C)
        assert abs(cur - a.score(ref, lc)) < 1e-13 and abs(new - a.score(ref, ln)) < 1e-13
    assert Acdc(m, clean, clean, MODE_PAHQ).pair_sender_policy(v, g.head(0, 0), R) == (0.0, 0.0)
    a32 = Acdc(m, clean, corrupt, MODE_ALL_FP32)
    r1, t1 = a32.sweep(1e-3)
    r2, t2 = a32.sweep_sender_policy(1e-3)
    assert (r1 == r2).all() and all(abs(x[2] - y[2]) < 1e-12 and x[4] == y[4] for x, y in zip(t1, t2))
    cur_s, new_s = a.pair_sender_policy(v, g.head(0, 1), g.empty_removed())
    assert cur_s == 0.0 and new_s > 0 and new_s != a.kl_edge(v, g.head(0, 1))
