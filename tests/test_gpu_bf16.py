"""bfloat16 for the components that are not attention heads (paper, Sec. "Selective Precision Allocation
Strategy"): the device with nonattn_bf16 against the oracle with the same option -- weight patterns and the
two row kernels bit for bit, per-edge values and states at the binding bound under both metrics, sweeps
decision by decision, exact zero for identical prompts -- with the attention heads still on their own grid."""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402
import synth                                        # noqa: E402
from oracle import bf16                             # noqa: E402
from oracle.acdc import Acdc, METRIC_LOGIT_DIFF     # noqa: E402
from fp32_spread import SpreadModel, kl_with_spread  # noqa: E402
from tolerance import check_kl_cases                # noqa: E402
from test_gpu_parity import Pair, compare_sweep, random_removed     # noqa: E402

pytestmark = pytest.mark.gpu
NAMES = ("cfg1_hi", "mid_hi", "midllama_hi")


@pytest.fixture(scope="module")
def pairs():
    out = {}
    for name in NAMES:
        shape, w, clean, corrupt = workloads.make(name)
        out[name] = Pair(shape, w, clean, corrupt, nonattn_bf16=True)
    yield out
    for pr in out.values():
        pr.close()


def test_weight_patterns_bit_exact(pairs):
    import paper_2510_23264_amd as P
    for name, pr in pairs.items():
        s, om, gm = pr.shape, pr.om, pr.gm
        for l in range(s.n_layers):
            if s.d_mlp:
                for which, nm in ((P.W_IN, "W_in"), (P.W_OUT, "W_out")) + (((P.W_GATE, "W_gate"),) if s.act == 2 else ()):
                    got = gm.get_weight_bf16(which, l, om.qc[nm][l].shape)
                    assert got.dtype == om.qc[nm].dtype == np.uint16 and np.array_equal(got, om.qc[nm][l]), (name, nm, l)
                    with pytest.raises(P.PahqError):
                        gm.get_weight_q(which, l, 0, om.qc[nm][l].shape)      # not e4m3 codes in this mode
            # the heads keep the e4m3 grid
            for h in range(s.n_heads):
                for which, nm in ((P.W_Q, "W_Q"), (P.W_O, "W_O")):
                    codes, scale = gm.get_weight_q(which, l, h, om.qc[nm][l, h].shape)
                    assert om.qc[nm].dtype == np.uint8 and scale == om.qs[nm][l, h] and (codes == om.qc[nm][l, h]).all()
        assert np.array_equal(gm.get_weight_bf16(P.W_U, 0, om.qc["W_U"].shape), om.qc["W_U"])


@pytest.mark.parametrize("site,cols_list", [(0, (64, 100, 320, 3072, 11008)), (1, (64, 128, 320, 768, 4096))])
def test_row_kernels_round_to_bfloat16_bit_exact(pairs, site, cols_list):
    gm = pairs["mid_hi"].gm
    rng = np.random.default_rng(21 + site)
    for cols in cols_list:
        x = (rng.standard_normal((23, cols)) * np.exp(rng.normal(size=(23, 1)) * 4)).astype(np.float32)
        x[3] = 0
        x[4, :] = np.float32(1e-30)
        n = min(cols, 60)
        x[5, :n] = (1.0 + (np.arange(n) + 0.5) * 2.0 ** -7).astype(np.float32)      # exact ties between neighbouring patterns
        x[6, :n] = -x[5, :n]
        got = gm.round_rows_bf16(x, site)
        assert np.array_equal(got, bf16.encode(x)), (site, cols, np.argwhere(got != bf16.encode(x))[:4])


@pytest.mark.parametrize("name", NAMES)
def test_edges_with_bfloat16_non_attention_components(pairs, name):
    pr = pairs[name]
    g = pr.g
    L, H = pr.shape.n_layers, pr.shape.n_heads
    receivers = [g.OUT, g.headin(L - 1, H - 1, 1), g.headin(0, 0, 2)] + ([g.mlpin(L - 1), g.mlpin(0)] if pr.shape.d_mlp else [])
    cases, got = [], []
    for i, r in enumerate(receivers):
        R = g.empty_removed() if i % 2 == 0 else random_removed(g, 0.4, 31 + i, from_receiver=r)
        senders = np.arange(g.n_upstream(r), dtype=np.int32)
        pr.gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
        got.append(np.concatenate([[pr.gm.eval_current(r)], pr.gm.eval_edges(r, senders)]))
        cases.append((r, R, senders))
    pr.gm.set_removed(np.zeros(g.n_edges(), np.uint8))
    res = kl_with_spread(pr.om, pr.clean, pr.corrupt, pr.mode, cases, seeds=4)
    want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
    sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
    worst = check_kl_cases(np.concatenate(got), want, sigma, what=name + " bf16 non-attention")
    print(name, "bf16 non-attention components: median KL %.3g, worst |d| / bound %.3f" % (np.median(want), worst))
    # the option is seen: the same cases with everything on the e4m3 grid give other values
    from oracle.model import Model
    o8 = Acdc(Model(pr.shape, pr.w), pr.clean, pr.corrupt, pr.mode)
    r, R, senders = cases[0]
    kl8 = np.array([o8.kl_edge(r, int(u), removed=R) for u in senders[:6]])
    assert (np.abs(kl8 - want[1:7]) > 10 * (1e-6 + 1e-3 * np.abs(kl8))).any()


def test_sweeps_with_bfloat16_non_attention_components(pairs):
    equal = 0
    for name, taus in (("cfg1_hi", (0.03,)), ("mid_hi", (0.01,)), ("midllama_hi", (0.03,))):
        for tau in taus:
            equal += compare_sweep(pairs[name], tau)[0] == "equal"
    assert equal >= 2


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi"])
def test_logit_difference_and_exact_zero(name):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    ans, dis = synth.make_answers(shape.vocab, B, "uniform", 78)
    om = SpreadModel(shape, w, nonattn_bf16=True)
    g = om.g
    margs = dict(metric=METRIC_LOGIT_DIFF, answer=ans, distractor=dis)
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8, nonattn_bf16=True)
    try:
        gm.set_metric(P.METRIC_LOGIT_DIFF, ans, dis)
        gm.clean_cache(clean, corrupt)
        cases = [(r, g.empty_removed(), list(range(g.n_upstream(r)))) for r in (g.OUT, g.headin(shape.n_layers - 1, 0, 0), g.mlpin(1))]
        res = kl_with_spread(om, clean, corrupt, 2, cases, seeds=4, **margs)
        got, want, sigma = [], [], []
        for (r, R, senders), o in zip(cases, res):
            got += [gm.eval_current(r)] + list(gm.eval_edges(r, np.array(senders, np.int32)))
            want += [o["kl_current"]] + o["kl_new"]
            sigma += [o["sigma_current"]] + o["sigma_new"]
        check_kl_cases(got, want, sigma, what=name + " logit difference, bf16 non-attention")
        # identical prompts, every node computed: exactly zero under both metrics
        for metric in (P.METRIC_LOGIT_DIFF, P.METRIC_KL):
            gm.set_metric(metric, ans, dis)
            gm.clean_cache(clean, clean.copy())
            gm.set_dead_node_skipping(False)
            for r in (g.OUT, g.mlpin(1), g.headin(2, 1, 0)):
                gm.set_removed(g.removed_to_flat(random_removed(g, 0.5, 3, from_receiver=r)).astype(np.uint8))
                assert (gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) == 0.0).all() and gm.eval_current(r) == 0.0
            gm.set_removed(np.zeros(g.n_edges(), np.uint8))
            gm.set_dead_node_skipping(True)
    finally:
        gm.close()
    with pytest.raises(P.PahqError):
        P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8, nonattn_bf16=True, mma=P.MMA_FP8)


# ------------------------------------------------------------------ the 16-bit point: the heads in bfloat16 as well
@pytest.fixture(scope="module")
def pairs16():
    out = {}
    for name in ("mid_hi", "midllama_hi"):
        shape, w, clean, corrupt = workloads.make(name)
        out[name] = Pair(shape, w, clean, corrupt, low_bits=16)
    yield out
    for pr in out.values():
        pr.close()


def test_sixteen_bits_weights_and_rows_bit_exact(pairs16):
    import paper_2510_23264_amd as P
    for name, pr in pairs16.items():
        s, om, gm = pr.shape, pr.om, pr.gm
        for l in range(s.n_layers):
            for h in range(s.n_heads):
                for which, nm in ((P.W_Q, "W_Q"), (P.W_K, "W_K"), (P.W_V, "W_V"), (P.W_O, "W_O")):
                    got = gm.get_weight_bf16(which, l, om.qc[nm][l, h].shape, head=h)
                    assert np.array_equal(got, om.qc[nm][l, h]), (name, nm, l, h)
            for which, nm in ((P.W_IN, "W_in"), (P.W_OUT, "W_out")):
                assert np.array_equal(gm.get_weight_bf16(which, l, om.qc[nm][l].shape), om.qc[nm][l]), (name, nm, l)
        with pytest.raises(P.PahqError):
            gm.get_weight_q(P.W_Q, 0, 0, om.qc["W_Q"][0, 0].shape)
        with pytest.raises(P.PahqError):
            gm.quantize_rows(np.zeros((2, 64), np.float32))
    gm = pairs16["mid_hi"].gm
    rng = np.random.default_rng(3)
    for cols in (16, 32, 64, 128):                                     # the attention kernel's output rounding
        x = (rng.standard_normal((19, cols)) * np.exp(rng.normal(size=(19, 1)) * 3)).astype(np.float32)
        x[2] = 0
        x[3, : min(cols, 16)] = (1.0 + (np.arange(min(cols, 16)) + 0.5) * 2.0 ** -7).astype(np.float32)
        assert np.array_equal(gm.round_rows_bf16(x, 2), bf16.encode(x)), cols


@pytest.mark.parametrize("name", ["mid_hi", "midllama_hi"])
def test_sixteen_bits_edges_and_sweeps(pairs16, name):
    pr = pairs16[name]
    g = pr.g
    L, H = pr.shape.n_layers, pr.shape.n_heads
    cases, got = [], []
    for i, r in enumerate((g.OUT, g.headin(L - 1, H - 1, 1), g.headin(0, 0, 2), g.mlpin(L - 1), g.headin(1, 0, 0))):
        R = g.empty_removed() if i % 2 == 0 else random_removed(g, 0.4, 71 + i, from_receiver=r)
        senders = np.arange(g.n_upstream(r), dtype=np.int32)
        pr.gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
        got.append(np.concatenate([[pr.gm.eval_current(r)], pr.gm.eval_edges(r, senders)]))
        cases.append((r, R, senders))
    pr.gm.set_removed(np.zeros(g.n_edges(), np.uint8))
    res = kl_with_spread(pr.om, pr.clean, pr.corrupt, pr.mode, cases, seeds=4)
    want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
    sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
    worst = check_kl_cases(np.concatenate(got), want, sigma, what=name + " at 16 bits")
    print(name, "16 bits: median KL %.3g, worst |d| / bound %.3f" % (np.median(want), worst))
    assert compare_sweep(pr, {"mid_hi": 0.01, "midllama_hi": 0.03}[name])[0] == "equal"


def test_sixteen_bits_exact_zero_and_limits():
    import paper_2510_23264_amd as P
    shape, w, clean, _ = workloads.make("midllama_hi")
    B, S = clean.shape
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8, low_bits=16)
    try:
        gm.clean_cache(clean, clean.copy())
        gm.set_dead_node_skipping(False)
        from oracle.graph import Graph
        g = Graph(shape.n_layers, shape.n_heads, True)
        for r in (g.OUT, g.mlpin(1), g.headin(2, 1, 0)):
            gm.set_removed(g.removed_to_flat(random_removed(g, 0.5, 3, from_receiver=r)).astype(np.uint8))
            assert (gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) == 0.0).all() and gm.eval_current(r) == 0.0
    finally:
        gm.close()
    small, w1, c1, _ = workloads.make("cfg1_hi")                        # heads of 16 values: no bfloat16 output projection
    with pytest.raises(P.PahqError) as e:
        P.Model(small, w1, c1.shape[0], c1.shape[1], low_bits=16)
    assert e.value.code == -6
