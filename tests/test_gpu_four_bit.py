"""The 4-bit point of the paper's bit-width ablation (Sec. "Ablation Studies", Different Quantization
Precisions; Appendix "Quantization", Eq. RTN-Q with N = 4) on the device against the oracle on the same
grid: weight multiples and steps and the three activation quantisers bit for bit, per-edge values at the
binding bound, sweeps decision by decision."""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402
from oracle import e4m3                             # noqa: E402
from oracle.rtn import Rtn                          # noqa: E402
from oracle.acdc import MODE_PAHQ, MODE_ALL_FP8     # noqa: E402
from fp32_spread import kl_with_spread              # noqa: E402
from tolerance import check_kl_cases                # noqa: E402
from test_gpu_parity import Pair, compare_sweep, random_removed     # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pairs():
    out = {}
    for name in ("cfg1_hi", "mid_hi", "midllama_hi"):
        shape, w, clean, corrupt = workloads.make(name)
        out[name] = Pair(shape, w, clean, corrupt, low_bits=4)
    yield out
    for pr in out.values():
        pr.close()


def test_weight_multiples_and_steps_bit_exact(pairs):
    import paper_2510_23264_amd as P
    for name, pr in pairs.items():
        s, om, gm = pr.shape, pr.om, pr.gm
        for l in range(s.n_layers):
            for h in range(s.n_heads):
                for which, nm in ((P.W_Q, "W_Q"), (P.W_K, "W_K"), (P.W_V, "W_V"), (P.W_O, "W_O")):
                    codes, step = gm.get_weight_q(which, l, h, om.qc[nm][l, h].shape)
                    assert step == om.qs[nm][l, h], (name, nm, l, h)
                    # the library stores the multiple as the e4m3 code of that integer
                    assert np.array_equal(e4m3.decode(codes), om.qc[nm][l, h].astype(np.float64)), (name, nm, l, h)
            if s.d_mlp:
                for which, nm in ((P.W_IN, "W_in"), (P.W_OUT, "W_out")) + (((P.W_GATE, "W_gate"),) if s.act == 2 else ()):
                    codes, step = gm.get_weight_q(which, l, 0, om.qc[nm][l].shape)
                    assert step == om.qs[nm][l] and np.array_equal(e4m3.decode(codes), om.qc[nm][l].astype(np.float64)), (name, nm, l)
        codes, step = gm.get_weight_q(P.W_U, 0, 0, om.qc["W_U"].shape)
        assert step == om.qs["W_U"] and np.array_equal(e4m3.decode(codes), om.qc["W_U"].astype(np.float64))
        assert np.abs(e4m3.decode(codes)).max() == 8.0


@pytest.mark.parametrize("site,cols_list", [(0, (64, 100, 320, 3072)), (1, (64, 128, 320, 768)), (2, (16, 32, 64, 128))])
def test_every_quantiser_site_is_bit_exact_at_four_bits(pairs, site, cols_list):
    gm = pairs["mid_hi"].gm
    q = Rtn(4)
    rng = np.random.default_rng(11 + site)
    for cols in cols_list:
        x = (rng.standard_normal((29, cols)) * rng.uniform(1e-4, 300, (29, 1))).astype(np.float32)
        x[3] = 0
        x[4, :] = np.float32(1e-30)
        n = min(cols, 16)
        x[5, :n] = (np.arange(n) + 0.5).astype(np.float32) * 0.5; x[5, 0] = 8.0      # step exactly 1: every tie of the grid
        x[6, :n] = -x[5, :n]
        codes, steps = gm.quantize_rows(x, site=site)
        k, st = q.quantize_rows(x)
        assert (steps.view(np.uint32) == st.view(np.uint32)).all(), (site, cols)
        assert np.array_equal(e4m3.decode(codes), k.astype(np.float64)), (site, cols)


@pytest.mark.parametrize("name", ["cfg1_hi", "mid_hi", "midllama_hi"])
def test_edges_at_four_bits(pairs, name):
    pr = pairs[name]
    g = pr.g
    L, H = pr.shape.n_layers, pr.shape.n_heads
    receivers = [g.OUT, g.headin(L - 1, H - 1, 1), g.headin(0, 0, 2)] + ([g.mlpin(L - 1)] if pr.shape.d_mlp else [])
    cases, got = [], []
    for i, r in enumerate(receivers):
        R = g.empty_removed() if i % 2 == 0 else random_removed(g, 0.4, 21 + i, from_receiver=r)
        senders = np.arange(g.n_upstream(r), dtype=np.int32)
        pr.gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
        got.append(np.concatenate([[pr.gm.eval_current(r)], pr.gm.eval_edges(r, senders)]))
        cases.append((r, R, senders))
    pr.gm.set_removed(np.zeros(g.n_edges(), np.uint8))
    res = kl_with_spread(pr.om, pr.clean, pr.corrupt, pr.mode, cases, seeds=4)
    want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
    sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
    worst = check_kl_cases(np.concatenate(got), want, sigma, what=name + " at 4 bits")
    print(name, "4-bit grid: median KL %.3g, worst |d| / bound %.3f" % (np.median(want), worst))
    # the grid is seen: the same cases on the e4m3 grid give other values
    from oracle.model import Model
    from oracle.acdc import Acdc
    o8 = Acdc(Model(pr.shape, pr.w), pr.clean, pr.corrupt, pr.mode)
    r, R, senders = cases[0]
    kl8 = np.array([o8.kl_edge(r, int(u), removed=R) for u in senders[:6]])
    assert (np.abs(kl8 - want[1:7]) > 10 * (1e-6 + 1e-3 * np.abs(kl8))).any()


def test_sweeps_at_four_bits(pairs):
    equal = 0
    for name, taus in (("cfg1_hi", (0.05, 0.3)), ("mid_hi", (0.01,))):
        for tau in taus:
            equal += compare_sweep(pairs[name], tau)[0] == "equal"
    assert equal >= 1


def test_clean_patch_is_exactly_zero_at_four_bits():
    import paper_2510_23264_amd as P
    shape, w, clean, _ = workloads.make("mid_hi")
    B, S = clean.shape
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8, low_bits=4)
    try:
        gm.clean_cache(clean, clean.copy())
        gm.set_dead_node_skipping(False)
        from oracle.graph import Graph
        g = Graph(shape.n_layers, shape.n_heads, shape.d_mlp > 0)
        for r in (g.OUT, g.mlpin(1), g.headin(2, 1, 0)):
            gm.set_removed(g.removed_to_flat(random_removed(g, 0.5, 3, from_receiver=r)).astype(np.uint8))
            assert (gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32)) == 0.0).all()
            assert gm.eval_current(r) == 0.0
    finally:
        gm.close()
