"""Sequences of 33 to 64 positions (three and four 16-position tiles in the attention kernel) against the oracle:
cached runs element by element in the all-fp32 mode, per-edge values at the binding bound under mixed precision,
learned and rotary positions."""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import synth                                        # noqa: E402
from synth import ModelShape                        # noqa: E402
from oracle.acdc import MODE_PAHQ                   # noqa: E402
from plain_forward import plain_forward             # noqa: E402
from fp32_spread import kl_with_spread              # noqa: E402
from tolerance import check_kl_cases                # noqa: E402
from test_gpu_parity import Pair, random_removed    # noqa: E402

pytestmark = pytest.mark.gpu

GPT = dict(n_layers=2, n_heads=3, d_head=32, d_model=64, d_mlp=128, vocab=300)
LLAMA = dict(n_layers=2, n_heads=2, d_head=64, d_model=128, d_mlp=192, vocab=257, norm=1, act=2, pos=1, norm_eps=1e-6)


@pytest.mark.parametrize("kind,S", [("gpt", 33), ("gpt", 41), ("gpt", 48), ("gpt", 64), ("llama", 40), ("llama", 64)])
def test_long_sequences(kind, S):
    import paper_2510_23264_amd as P
    shape = ModelShape(n_ctx=S, **(GPT if kind == "gpt" else LLAMA))
    w = synth.make_weights(shape, 11, std=0.25 if kind == "gpt" else 0.12, affine_std=0.1)
    clean, corrupt = synth.make_tokens(shape.vocab, 3, S, "uniform", 5, False, 13)
    B = clean.shape[0]
    # nothing quantised: logits of the cached clean run against a textbook forward
    gm = P.Model(shape, w, B, S, precision=P.ALL_FP32, max_batch_edges=4)
    try:
        gm.clean_cache(clean, corrupt)
        want = plain_forward(shape, w, clean)
        got = gm.get_logits(0)
        assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max(), (kind, S, np.abs(got - want).max() / np.abs(want).max())
    finally:
        gm.close()
    pr = Pair(shape, w, clean, corrupt, max_batch=4)
    try:
        g = pr.g
        cases, got = [], []
        for i, r in enumerate((g.OUT, g.headin(1, 1, 0), g.headin(1, 0, 2), g.mlpin(0), g.headin(0, 0, 1))):
            R = g.empty_removed() if i % 2 == 0 else random_removed(g, 0.4, 51 + i, from_receiver=r)
            senders = np.arange(g.n_upstream(r), dtype=np.int32)
            pr.gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
            got.append(np.concatenate([[pr.gm.eval_current(r)], pr.gm.eval_edges(r, senders)]))
            cases.append((r, R, senders))
        res = kl_with_spread(pr.om, clean, corrupt, MODE_PAHQ, cases, seeds=3)
        want = np.concatenate([[r["kl_current"]] + list(r["kl_new"]) for r in res])
        sigma = np.concatenate([[r["sigma_current"]] + list(r["sigma_new"]) for r in res])
        worst = check_kl_cases(np.concatenate(got), want, sigma, what="%s S=%d" % (kind, S))
        print(kind, "S", S, "median KL %.3g, worst |d| / bound %.3f" % (np.median(want), worst))
        assert np.median(want) > 1e-3
    finally:
        pr.close()


def test_limits():
    import paper_2510_23264_amd as P
    shape = ModelShape(n_ctx=65, **GPT)
    with pytest.raises(P.PahqError) as e:
        P.workspace_bytes(P.Config.from_shape(shape), 2, 65)
    assert e.value.code == -6
    wide = ModelShape(n_layers=1, n_heads=1, d_head=128, d_model=128, d_mlp=0, vocab=50, n_ctx=40, act=0)
    with pytest.raises(P.PahqError) as e:
        P.workspace_bytes(P.Config.from_shape(wide), 2, 40)      # 128-wide heads: up to 32 positions
    assert e.value.code == -6
    assert P.workspace_bytes(P.Config.from_shape(wide), 2, 32) > 0
