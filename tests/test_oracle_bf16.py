"""Pins of oracle/bf16.py and of the oracle's forward with bfloat16 non-attention components (paper, Sec.
"Selective Precision Allocation Strategy")."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
from oracle import bf16                               # noqa: E402
from oracle.model import Model, ALL                   # noqa: E402
from loop_forward import loop_forward                 # noqa: E402
from test_oracle_model import tiny, TINY_GELU, TINY_LLAMA, TINY_ATTN, _names, _rel     # noqa: E402


def test_format_closed_form():
    # 1 sign, 8 exponent (bias 127), 7 mantissa bits: value = (-1)^s 2^(e-127) (1 + m/128); subnormals m/128 2^-126
    for code, val in ((0x3F80, 1.0), (0x3F81, 1.0 + 2.0 ** -7), (0x4000, 2.0), (0xC040, -3.0), (0x0000, 0.0),
                      (0x0080, 2.0 ** -126), (0x0001, 2.0 ** -133), (0x7F7F, (2 - 2.0 ** -7) * 2.0 ** 127)):
        assert bf16.decode(np.array([code], np.uint16))[0] == val, hex(code)
    # every finite pattern decodes by the closed form, and encoding its value gives the pattern back
    codes = np.arange(0x10000, dtype=np.uint32)
    codes = codes[(codes & 0x7F80) != 0x7F80].astype(np.uint16)
    s = np.where(codes & 0x8000, -1.0, 1.0)
    e = ((codes >> 7) & 0xFF).astype(np.int64)
    m = (codes & 0x7F).astype(np.float64)
    want = np.where(e == 0, s * m / 128.0 * 2.0 ** -126, s * (1 + m / 128.0) * 2.0 ** (e - 127.0))
    got = bf16.decode(codes)
    assert np.array_equal(got, want)
    back = bf16.encode(got.astype(np.float32))
    assert np.array_equal(back, codes)                                # (-0 keeps its sign bit: 0x8000)


def test_nearest_and_ties():
    # ties between neighbours go to the even mantissa; just above / below a tie goes to the nearer one
    one = np.float32(1.0)
    step = np.float32(2.0 ** -7)
    assert bf16.decode(bf16.encode(np.array([one + step / 2], np.float32)))[0] == 1.0                      # tie -> even (m = 0)
    assert bf16.decode(bf16.encode(np.array([one + step + step / 2], np.float32)))[0] == 1.0 + 2 * step    # tie -> even (m = 2)
    assert bf16.decode(bf16.encode(np.array([np.nextafter(one + step / 2, np.float32(2))], np.float32)))[0] == 1.0 + step
    assert bf16.decode(bf16.encode(np.array([np.nextafter(one + step / 2, np.float32(0))], np.float32)))[0] == 1.0
    # brute force over a binade: the chosen pattern is a nearest one among all patterns
    rng = np.random.default_rng(0)
    x = (rng.uniform(1, 2, 2000) * rng.choice([-1, 1], 2000) * 2.0 ** rng.integers(-20, 20, 2000)).astype(np.float32)
    got = bf16.decode(bf16.encode(x))
    assert (np.abs(got - x) <= np.abs(x) * 2.0 ** -8).all()            # half a unit in the last of 8 significand bits
    grid = bf16.decode(np.arange(0x3F80, 0x4001, dtype=np.uint16))   # all values in [1, 2]
    y = rng.uniform(1, 2, 500).astype(np.float32)
    near = grid[np.abs(grid[None, :] - y[:, None].astype(np.float64)).argmin(axis=1)]
    g = bf16.decode(bf16.encode(y))
    assert (np.abs(g - y) <= np.abs(near - y) + 0).all()
    with pytest.raises(ValueError):
        bf16.encode(np.array([np.inf], np.float32))
    with pytest.raises(ValueError):
        bf16.encode(np.array([3.4e38], np.float32))                    # rounds past the largest finite value


def test_against_a_library_conversion():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(20000) * np.exp(rng.normal(size=20000) * 8)).astype(np.float32)
    x[:4] = [0.0, -0.0, 1e-40, -1e-39]                                  # zeros and binary32 subnormals
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    assert np.array_equal(bf16.decode(bf16.encode(x)), want)
    codes, scale = bf16.quantize_rows(x.reshape(100, 200))
    assert codes.dtype == np.uint16 and scale.shape == (100,) and (scale == 1).all()
    c2, s2 = bf16.quantize_groups(x.reshape(100, 200), axis=None)
    assert np.array_equal(c2, codes) and s2 == 1.0


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA, TINY_ATTN])
def test_forward_with_bfloat16_non_attention_components(shape):
    """With nonattn_bf16 the MLP matrices and the unembedding multiply bfloat16-rounded operands, the attention
    heads keep their grid: equal to the independent loop forward handed the two quantisers; leaving the
    bfloat16 rounding out of any one non-attention operand, or putting it on an attention operand, is seen."""
    from oracle import e4m3
    m8, w, clean, _ = tiny(shape, B=2)
    mb = Model(shape, w, nonattn_bf16=True)
    snd, _ = _names(mb.g)
    for pi in (frozenset(), frozenset([(1, 0)])):
        outs, lg = mb.forward(clean, pi)
        l_out, l_lg = loop_forward(shape, w, clean, pi=pi, codec=e4m3, codec_other=bf16)
        assert _rel(lg, l_lg) < 1e-12, sorted(pi)
        for s, nm in snd.items():
            assert _rel(outs[s].reshape(l_out[nm].shape), l_out[nm]) < 1e-12, (sorted(pi), nm)
    _, lg = mb.forward(clean, frozenset())
    sites = ["act:u", "w:u"] + (["act:in", "w:in", "act:out", "w:out"] if shape.d_mlp else []) + (["w:gate"] if shape.act == 2 else [])
    for site in sites:
        _, l_lg = loop_forward(shape, w, clean, codec=e4m3, codec_other=bf16, drop=site)
        assert _rel(lg, l_lg) > 1e-9, site
    _, l_lg = loop_forward(shape, w, clean, codec=bf16, codec_other=bf16)          # attention heads in bfloat16 too
    assert _rel(lg, l_lg) > 1e-7
    _, lg8 = m8.forward(clean, frozenset())
    assert _rel(lg, lg8) > 1e-7                                                     # not the all-e4m3 forward
    _, full = mb.forward(clean, ALL)
    _, full8 = m8.forward(clean, ALL)
    assert np.array_equal(full, full8)                                              # nothing quantised: no grid matters
    # with every head in fp32 only the non-attention products are rounded: bfloat16 (8 significand bits, no
    # shared scale) stays closer to the unquantised run than e4m3 (4 significand bits)
    heads = frozenset((l, h) for l in range(shape.n_layers) for h in range(shape.n_heads))
    _, a = mb.forward(clean, heads)
    _, b = m8.forward(clean, heads)
    assert np.abs(a - full).max() < 0.5 * np.abs(b - full).max()


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA])
def test_forward_at_sixteen_bits(shape):
    """low_bits = 16 (the 16-bit point of the paper's bit-width table): every quantised operand, the heads' included,
    is rounded to bfloat16 -- equal to the loop forward handed that one quantiser for everything, and closer to the
    unquantised run than the 8-bit forward (8 significand bits against 4)."""
    m8, w, clean, _ = tiny(shape, B=2)
    m16 = Model(shape, w, low_bits=16)
    snd, _ = _names(m16.g)
    for pi in (frozenset(), frozenset([(0, 1)])):
        outs, lg = m16.forward(clean, pi)
        l_out, l_lg = loop_forward(shape, w, clean, pi=pi, codec=bf16, codec_other=bf16)
        assert _rel(lg, l_lg) < 1e-12, sorted(pi)
        for s, nm in snd.items():
            assert _rel(outs[s].reshape(l_out[nm].shape), l_out[nm]) < 1e-12, (sorted(pi), nm)
    _, full = m16.forward(clean, ALL)
    _, lg16 = m16.forward(clean, frozenset())
    _, lg8 = m8.forward(clean, frozenset())
    assert np.abs(lg16 - full).max() < 0.25 * np.abs(lg8 - full).max()
    assert np.array_equal(m16.forward(clean, frozenset())[1], Model(shape, w, low_bits=16, nonattn_bf16=True).forward(clean, frozenset())[1])
