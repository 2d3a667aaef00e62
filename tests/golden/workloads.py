"""Recipes of the workloads that have stored expected values (shared by the script that writes them and
by the GPU tests that rebuild the same inputs; synth only, no arithmetic of the method).

Two kinds.  The named configurations as they are specified (weights N(0, 0.02^2), few resampled
positions): their KLs are small, mostly below 1e-3.  And '_hi' variants of the same shapes with a larger
weight scale and more resampled positions, so that candidate KLs are O(0.01 .. 1) and the relative part
of the parity bound governs."""
import numpy as np

import synth
from synth import ModelShape

MID = ModelShape(n_layers=3, n_heads=4, d_head=32, d_model=128, d_mlp=320, vocab=1000, n_ctx=12)
MID_LLAMA = ModelShape(n_layers=3, n_heads=2, d_head=64, d_model=128, d_mlp=200, vocab=777, n_ctx=10,
                       norm=1, act=2, pos=1, norm_eps=1e-6)

# name -> (config or shape, weight std, affine std, resampled positions k (None = the config's), B, seed)
RECIPES = {
    "cfg1_hi": ("cfg1", 0.5, 0.05, None, None, None),
    "mid_hi": (MID, 0.08, 0.05, 8, 6, 11),
    "mid_hi2": (MID, 0.3, 0.05, 3, 6, 11),
    "midllama_hi": (MID_LLAMA, 0.08, 0.05, 8, 6, 12),
    "midllama_hi2": (MID_LLAMA, 0.3, 0.05, 3, 6, 12),
    "cfg2": ("cfg2", 0.02, 0.0, None, None, None),
    "cfg2_hi": ("cfg2", 0.06, 0.0, 16, None, None),
    "cfg3": ("cfg3", 0.02, 0.0, None, None, None),
    "cfg3_hi": ("cfg3", 0.05, 0.0, 14, None, None),
    "cfg4": ("cfg4", 0.02, 0.0, None, None, None),
    "cfg5_L2": ("cfg5_L2", 0.02, 0.0, None, None, None),
    "cfg5_L8": ("cfg5_L8", 0.02, 0.0, None, None, None),
}


def make(name):
    """(shape, weights, clean, corrupt) of a named recipe."""
    base, std, affine, k, B, seed = RECIPES[name]
    if isinstance(base, str):
        spec = synth.CONFIGS[base]
        shape = synth.make_shape(base)
        w = synth.make_weights(shape, spec["seed"], std=std, affine_std=affine)
        clean, corrupt = synth.make_tokens(shape.vocab, spec["B"], spec["S"], spec["law"],
                                           spec["k"] if k is None else k, spec["shared_pos"], spec["seed"])
    else:
        shape = base
        w = synth.make_weights(shape, seed, std=std, affine_std=affine)
        clean, corrupt = synth.make_tokens(shape.vocab, B, shape.n_ctx, "uniform", k, False, seed)
    return shape, w, clean, corrupt


def removed_rows(n_receivers, n_upstream, frac, seed, from_receiver):
    """The removed set of a case, as one boolean row per receiver: every in-edge of every receiver >=
    from_receiver removed with probability frac (a state the sweep can be in when it reaches that
    receiver); frac = 0 is the empty set.  n_upstream: callable receiver -> number of in-edges."""
    rng = np.random.default_rng(seed)
    rows = []
    for r in range(n_receivers):
        n_up = n_upstream(r)
        if frac > 0 and r >= from_receiver:
            rows.append(rng.random(n_up) < frac)
        else:
            rows.append(np.zeros(n_up, dtype=bool))
    return rows
