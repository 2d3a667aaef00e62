"""Seeded synthetic workloads.

The paper measures on trained checkpoints (GPT-2 small and two small
interpretability models) with templated prompt pairs that differ in a few
name positions (Experiment section; appendix "Models and Datasets").  None of
those assets are available offline, so every workload here is a stand-in with
the same shapes: random-initialised weights and token batches whose corrupt
copy differs from the clean one in a handful of positions.

Array layouts (all float32, C-contiguous) -- the same for every consumer:

  W_E   [vocab][d_model]            W_pos [n_ctx][d_model]   (learned positions only)
  W_Q/W_K/W_V [L][H][d_model][d_head]     b_Q/b_K/b_V [L][H][d_head]
  W_O   [L][H][d_head][d_model]           b_O  [L][d_model]
  ln1_g/ln1_b/ln2_g/ln2_b [L][d_model]    lnf_g/lnf_b [d_model]
  W_in  [L][d_model][d_mlp]   b_in [L][d_mlp]   W_gate [L][d_model][d_mlp] (SwiGLU only)
  W_out [L][d_mlp][d_model]   b_out [L][d_model]
  W_U   [d_model][vocab]      b_U [vocab]
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np

NORM_LAYER, NORM_RMS = 0, 1
ACT_NONE, ACT_GELU, ACT_SWIGLU = 0, 1, 2
POS_LEARNED, POS_ROPE = 0, 1


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    n_heads: int
    d_head: int
    d_model: int
    d_mlp: int          # 0 = attention-only
    vocab: int
    n_ctx: int
    norm: int = NORM_LAYER
    act: int = ACT_GELU
    pos: int = POS_LEARNED
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0

    def as_dict(self):
        return asdict(self)


# name -> (shape kwargs, batch B, seq S, token law, resampled positions k,
#          shared positions?, tau list, receiver sample size (0 = all), seed)
CONFIGS = {
    "cfg1": dict(shape=dict(n_layers=2, n_heads=4, d_head=16, d_model=64, d_mlp=0, vocab=512,
                            n_ctx=16, act=ACT_NONE),
                 B=8, S=16, law="uniform", k=3, shared_pos=False, taus=(0.01,), n_recv=0, seed=101),
    "cfg2": dict(shape=dict(n_layers=4, n_heads=8, d_head=64, d_model=512, d_mlp=2048, vocab=8192,
                            n_ctx=32),
                 B=32, S=32, law="uniform", k=4, shared_pos=False, taus=(0.01,), n_recv=0, seed=202),
    "cfg3": dict(shape=dict(n_layers=12, n_heads=12, d_head=64, d_model=768, d_mlp=3072, vocab=50257,
                            n_ctx=16),
                 B=50, S=16, law="zipf", k=2, shared_pos=True, taus=(0.005, 0.02, 0.05), n_recv=0,
                 seed=303),
    "cfg4": dict(shape=dict(n_layers=24, n_heads=16, d_head=64, d_model=1024, d_mlp=4096, vocab=50257,
                            n_ctx=24),
                 B=64, S=24, law="zipf", k=3, shared_pos=True, taus=(0.01,), n_recv=128, seed=404),
    "cfg5": dict(shape=dict(n_layers=32, n_heads=32, d_head=128, d_model=4096, d_mlp=11008, vocab=32000,
                            n_ctx=32, norm=NORM_RMS, act=ACT_SWIGLU, pos=POS_ROPE, norm_eps=1e-6),
                 B=16, S=32, law="zipf", k=4, shared_pos=True, taus=(0.01,), n_recv=64, seed=505),
    # cfg5's layer shape, batch and tokens at depth 2: small enough for a CPU check of every
    # kernel shape cfg5 launches (depth only repeats them)
    "cfg5_L2": dict(shape=dict(n_layers=2, n_heads=32, d_head=128, d_model=4096, d_mlp=11008, vocab=32000,
                               n_ctx=32, norm=NORM_RMS, act=ACT_SWIGLU, pos=POS_ROPE, norm_eps=1e-6),
                    B=16, S=32, law="zipf", k=4, shared_pos=True, taus=(0.01,), n_recv=0, seed=506),
    # the same at depth 8: the deepest stack of cfg5 layers the CPU check handles in about an hour
    "cfg5_L8": dict(shape=dict(n_layers=8, n_heads=32, d_head=128, d_model=4096, d_mlp=11008, vocab=32000,
                               n_ctx=32, norm=NORM_RMS, act=ACT_SWIGLU, pos=POS_ROPE, norm_eps=1e-6),
                    B=16, S=32, law="zipf", k=4, shared_pos=True, taus=(0.01,), n_recv=0, seed=508),
}


def make_shape(name: str) -> ModelShape:
    return ModelShape(**CONFIGS[name]["shape"])


def _normal(rng, shape, std):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def make_weights(shape: ModelShape, seed: int, std: float = 0.02, affine_std: float = 0.0):
    """Random-initialised weights.  Matrices and embeddings ~ N(0, std^2).

    affine_std = 0 gives the benchmark recipe (biases 0, norm gains 1, norm
    offsets 0).  affine_std > 0 draws biases and norm offsets ~ N(0,
    affine_std^2) and gains ~ 1 + N(0, affine_std^2): used by tests so that
    no term of the model is trivially absent.
    """
    rng = np.random.default_rng(seed)
    L, H, dh, d, m, V = (shape.n_layers, shape.n_heads, shape.d_head, shape.d_model,
                         shape.d_mlp, shape.vocab)
    w = {}
    w["W_E"] = _normal(rng, (V, d), std)
    if shape.pos == POS_LEARNED:
        w["W_pos"] = _normal(rng, (shape.n_ctx, d), std)
    for nm in ("W_Q", "W_K", "W_V"):
        w[nm] = _normal(rng, (L, H, d, dh), std)
    w["W_O"] = _normal(rng, (L, H, dh, d), std)
    if m > 0:
        w["W_in"] = _normal(rng, (L, d, m), std)
        if shape.act == ACT_SWIGLU:
            w["W_gate"] = _normal(rng, (L, d, m), std)
        w["W_out"] = _normal(rng, (L, m, d), std)
    w["W_U"] = _normal(rng, (d, V), std)

    def aff(shp, base):
        if affine_std > 0:
            return (base + _normal(rng, shp, affine_std)).astype(np.float32)
        return np.full(shp, base, dtype=np.float32)

    for nm in ("b_Q", "b_K", "b_V"):
        w[nm] = aff((L, H, dh), 0.0)
    w["b_O"] = aff((L, d), 0.0)
    w["ln1_g"] = aff((L, d), 1.0)
    w["ln1_b"] = aff((L, d), 0.0)
    if m > 0:
        w["ln2_g"] = aff((L, d), 1.0)
        w["ln2_b"] = aff((L, d), 0.0)
        w["b_in"] = aff((L, m), 0.0)
        w["b_out"] = aff((L, d), 0.0)
    w["lnf_g"] = aff((d,), 1.0)
    w["lnf_b"] = aff((d,), 0.0)
    w["b_U"] = aff((V,), 0.0)
    if shape.norm == NORM_RMS:          # RMSNorm has no offset
        for nm in ("ln1_b", "ln2_b", "lnf_b"):
            if nm in w:
                w[nm][...] = 0.0
    return w


def _draw_tokens(rng, law, vocab, size):
    if law == "uniform":
        return rng.integers(0, vocab, size=size, dtype=np.int64).astype(np.int32)
    # Zipf(1.1) over ranks 1..V, rank r -> id r-1
    p = np.arange(1, vocab + 1, dtype=np.float64) ** -1.1
    cdf = np.cumsum(p / p.sum())
    u = rng.random(size=size)
    return np.minimum(np.searchsorted(cdf, u), vocab - 1).astype(np.int32)


def make_tokens(vocab: int, B: int, S: int, law: str, k: int, shared_pos: bool, seed: int):
    """Clean batch [B][S] and a corrupt copy with k positions resampled.

    The resampled token is forced to differ from the clean one.  The last
    position is never resampled.  shared_pos=True resamples the same k
    positions (drawn once from [1, S-2]) in every sequence, like the name
    slots of a prompt template; otherwise k positions per sequence are drawn
    from [0, S-2].
    """
    rng = np.random.default_rng(seed + 7919)
    clean = _draw_tokens(rng, law, vocab, (B, S))
    corrupt = clean.copy()
    if shared_pos:
        pos_all = np.tile(np.sort(rng.choice(np.arange(1, S - 1), size=k, replace=False)), (B, 1))
    else:
        pos_all = np.stack([np.sort(rng.choice(np.arange(0, S - 1), size=k, replace=False))
                            for _ in range(B)])
    for b in range(B):
        for p in pos_all[b]:
            t = clean[b, p]
            while t == clean[b, p]:
                t = _draw_tokens(rng, law, vocab, ())
            corrupt[b, p] = t
    return clean, corrupt


def make_answers(vocab: int, B: int, law: str, seed: int):
    """One answer and one distractor token id per sequence (different from each other), for the
    logit-difference task metric: stand-ins for the correct and the wrong name of a templated prompt."""
    rng = np.random.default_rng(seed + 15485863)
    ans = _draw_tokens(rng, law, vocab, (B,))
    dis = ans.copy()
    for b in range(B):
        while dis[b] == ans[b]:
            dis[b] = _draw_tokens(rng, law, vocab, ())
    return ans.astype(np.int32), dis.astype(np.int32)


def make_receiver_sample(n_receivers: int, count: int, seed: int):
    """Receiver ids drawn without replacement (all of them when count = 0)."""
    if count <= 0 or count >= n_receivers:
        return np.arange(n_receivers, dtype=np.int32)
    rng = np.random.default_rng(seed + 104729)
    return np.sort(rng.choice(n_receivers, size=count, replace=False)).astype(np.int32)


def make_workload(name: str, affine_std: float = 0.0):
    """(shape, weights, clean tokens, corrupt tokens, spec dict) for a named config."""
    spec = CONFIGS[name]
    shape = make_shape(name)
    w = make_weights(shape, spec["seed"], affine_std=affine_std)
    clean, corrupt = make_tokens(shape.vocab, spec["B"], spec["S"], spec["law"], spec["k"],
                                 spec["shared_pos"], spec["seed"])
    return shape, w, clean, corrupt, spec
