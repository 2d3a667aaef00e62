"""Pins for the oracle's e4m3 codec and quantiser (CPU only)."""
import json
import os
import numpy as np
import pytest
import torch

from oracle import e4m3

FACTS = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))


def test_decode_matches_paper_format():
    t = e4m3.decode_table()
    # smallest normal = 2^-6 (the paper's "minimum quantization step size")
    assert t[0x08] == 2.0 ** FACTS["e4m3_min_normal_step_log2"]["value"]
    assert t[0x7E] == 448.0 and np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    assert t[0x01] == 2.0 ** -9 and t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    # 4 exponent bits x 3 mantissa bits: spacing doubles every 8 codes above the subnormals
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()
    for e in range(1, 15):
        seg = pos[8 * e: 8 * e + 9] if e < 15 else pos[8 * e:]
        assert np.allclose(np.diff(seg), 2.0 ** (e - 7) / 8, rtol=0, atol=0)


def test_decode_matches_library_e4m3fn():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = e4m3.decode_table()
    fin = ~np.isnan(ours)
    assert (np.isnan(lib) == np.isnan(ours)).all()
    assert (lib[fin] == ours[fin]).all()


def test_encode_roundtrip_midpoints_saturation():
    t = e4m3.decode_table()
    codes = np.array([c for c in range(256) if not np.isnan(t[c])], dtype=np.uint8)
    assert (e4m3.encode(t[codes].astype(np.float32)) == codes).all()        # incl. -0 -> 0x80
    pos = t[:0x7F]
    mid = ((pos[1:] + pos[:-1]) / 2).astype(np.float32)                      # exact in binary32
    got = e4m3.encode(mid)
    lo = np.arange(0, 0x7E)
    expect = np.where(lo % 2 == 0, lo, lo + 1)                               # tie -> even code
    assert (got == expect).all()
    up = np.nextafter(mid, np.float32(np.inf))
    dn = np.nextafter(mid, np.float32(-np.inf))
    assert (e4m3.encode(up) == lo + 1).all() and (e4m3.encode(dn) == lo).all()
    assert (e4m3.encode(np.float32([448, 449, 464, 480, 1e30, np.inf])) == 0x7E).all()
    assert (e4m3.encode(np.float32([-449, -1e30])) == 0xFE).all()
    with pytest.raises(ValueError):
        e4m3.encode(np.float32([np.nan]))


def test_encode_matches_library_in_range():
    rng = np.random.default_rng(0)
    y = np.concatenate([rng.standard_normal(200000) * s for s in (1e-3, 1e-2, 1, 30, 150)]).astype(np.float32)
    y = y[np.abs(y) <= 448]
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert (e4m3.encode(y) == lib).all()


def test_mantissa_loss_example():
    """Paper, 'Mantissa Loss': a sum keeps nothing of the smaller addend once the
    exponents differ by 3 or more (3 mantissa bits)."""
    gap = FACTS["mantissa_loss_exponent_gap"]["value"]
    big = np.float32(1.0)
    for e in range(gap + 1, 8):                     # strictly below half an ulp (2^-4): absorbed
        small = np.float32(2.0 ** -e) * np.float32(1.75)
        if small < 2.0 ** -4:
            assert e4m3.decode(e4m3.encode(np.float32([big + small])))[0] == 1.0
    # gap of exactly 3 with mantissa 000: half an ulp -> tie -> even -> still lost
    assert e4m3.decode(e4m3.encode(np.float32([1.0 + 2.0 ** -(gap + 1)])))[0] == 1.0
    # gap 2 survives
    assert e4m3.decode(e4m3.encode(np.float32([1.0 + 2.0 ** -2])))[0] == 1.25


def test_quantiser_scale_and_codes():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((64, 96)) * rng.uniform(1e-3, 50, (64, 1))).astype(np.float32)
    x[5] = 0
    x[6, 3] = -np.abs(x[6]).max() * 2            # a negative extreme
    codes, s = e4m3.quantize_rows(x)
    assert codes.dtype == np.uint8 and s.dtype == np.float32
    amax = np.abs(x).max(axis=1)
    assert s[5] == 1.0 and (codes[5] == 0).all()
    nz = amax > 0
    assert (s[nz] == (amax[nz] / np.float32(448)).astype(np.float32)).all()
    # the absmax element lands on the top of the grid
    j = np.abs(x).argmax(axis=1)
    top = codes[np.arange(64), j] & 0x7F
    assert (top[nz] == 0x7E).all() and codes[6, 3] == 0xFE
    # error bound: half a grid step relative 2^-4, or half the subnormal step
    err = np.abs(e4m3.dequantize(codes, s) - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, s[:, None] * 2.0 ** -10) * (1 + 1e-6)
    assert (err <= bound).all()
    # re-quantising the dequantised values reproduces the codes
    c2, s2 = e4m3.quantize_rows(e4m3.dequantize(codes, s).astype(np.float32))
    assert (s2 == s).all() and (c2 == codes).all()
    # one scale for a whole tensor
    ct, st = e4m3.quantize_groups(x, axis=None)
    assert st == np.float32(np.abs(x).max() / np.float32(448))


def test_products_of_codes_exact_in_binary32():
    """Two e4m3 values have 4 significant bits each, so their product is exact in
    binary32 and the fp64 sum over codes is the exact GEMM result."""
    t = e4m3.decode_table()[:0x7F]
    p64 = np.outer(t, t)
    assert (p64.astype(np.float32).astype(np.float64) == p64).all()
