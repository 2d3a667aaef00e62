"""Pins of oracle/rtn.py (the 4-bit point of the paper's bit-width ablation: Appendix "Quantization",
Eq. RTN-Q with N = 4) and of the oracle's forward on that grid."""
import os
import sys
from fractions import Fraction

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
from oracle.rtn import Rtn                         # noqa: E402
from oracle.model import Model, ALL                # noqa: E402
from loop_forward import loop_forward              # noqa: E402
from test_oracle_model import tiny, TINY_GELU, TINY_LLAMA, _names, _rel     # noqa: E402


def test_grid_closed_forms():
    q = Rtn(4)
    rng = np.random.default_rng(0)
    x = rng.normal(size=(50, 37)).astype(np.float32) * rng.lognormal(size=(50, 1)).astype(np.float32)
    k, step = q.quantize_rows(x)
    amax = np.abs(x).max(axis=1)
    assert np.array_equal(step, amax / np.float32(8.0))            # step = max|x| / 2^(N-1), exact (a power of two)
    assert k.dtype == np.int16 and k.min() >= -8 and k.max() <= 8     # the multiples -2^(N-1) .. 2^(N-1)
    top = np.abs(x).argmax(axis=1)
    assert (np.abs(k[np.arange(50), top]) == 8).all()                # the largest magnitude sits on the top multiple
    assert np.array_equal(np.sign(k[k != 0]), np.sign(x[k != 0]))
    # a zero row: step 1, all multiples 0
    k0, s0 = q.quantize_rows(np.zeros((1, 5), np.float32))
    assert s0[0] == 1.0 and not k0.any()
    # N bits: 2^(N-1) steps from 0 to the maximum, for every N the formula is used with
    for bits in (2, 3, 4, 8):
        kk, ss = Rtn(bits).quantize_groups(np.array([1.0, -0.3, 0.0], np.float32), axis=None)
        assert ss == np.float32(1.0 / 2 ** (bits - 1)) and kk[0] == 2 ** (bits - 1)


def test_ties_go_to_even():
    q = Rtn(4)
    x = np.array([[8.0, 0.5, 1.5, 2.5, -2.5, 3.5, -0.5, 6.5, 7.5, -7.5]], np.float32)     # max 8 -> step exactly 1
    k, step = q.quantize_rows(x)
    assert step[0] == 1.0
    assert k[0].tolist() == [8, 0, 2, 2, -2, 4, 0, 6, 8, -8]


def test_against_exact_fractions_and_python_rounding():
    """Every multiple equals Python's round-half-even of the binary32 product x * inv, the product formed
    exactly in binary64 (24 + 24 significant bits) and rounded once; inv is the correctly rounded binary32
    reciprocal of the step (checked in exact rational arithmetic)."""
    q = Rtn(4)
    rng = np.random.default_rng(1)
    x = (rng.normal(size=(40, 33)) * np.exp(rng.normal(size=(40, 1)) * 3)).astype(np.float32)
    k, step = q.quantize_rows(x)
    for r in range(x.shape[0]):
        st = float(step[r])
        inv = np.float32(np.float32(1.0) / np.float32(st))
        exact = Fraction(1) / Fraction(st)
        ulp = Fraction(float(np.spacing(inv)))
        assert abs(Fraction(float(inv)) - exact) <= ulp / 2           # correctly rounded reciprocal
        for c in range(x.shape[1]):
            y = np.float32(float(x[r, c]) * float(inv))               # exact in binary64, one rounding to binary32
            assert int(k[r, c]) == round(float(y)), (r, c)


def test_half_step_error_bound_and_idempotence():
    q = Rtn(4)
    rng = np.random.default_rng(2)
    x = rng.normal(size=(64, 100)).astype(np.float32)
    k, step = q.quantize_rows(x)
    deq = q.decode(k) * step.astype(np.float64)[:, None]
    assert (np.abs(deq - x) <= 0.5 * step[:, None] * (1 + 2.0 ** -20)).all()
    assert (np.abs(deq - x).max(axis=1) > 0.3 * step).all()           # ... and the bound is not slack by much
    k2, step2 = q.quantize_rows(deq.astype(np.float32))
    assert np.array_equal(k, k2) and np.array_equal(step, step2)       # grid points are fixed points
    # one group for a whole matrix: the weight-slice form
    kw, sw = q.quantize_groups(x, axis=None)
    assert sw == np.float32(np.abs(x).max() / np.float32(8.0)) and np.abs(kw).max() == 8


@pytest.mark.parametrize("shape", [TINY_GELU, TINY_LLAMA])
def test_forward_on_the_four_bit_grid(shape):
    """The oracle's forward with low_bits = 4 equals the independent loop forward handed the 4-bit quantiser
    (same placement as at 8 bits, another grid); with nothing quantised the grid does not matter; and 4 bits
    are far coarser than 8 (the reason the paper calls them unusable)."""
    m8, w, clean, _ = tiny(shape, B=2)
    m4 = Model(shape, w, low_bits=4)
    snd, _ = _names(m4.g)
    for pi in (frozenset(), frozenset([(1, 0)]), frozenset([(0, 0), (1, 1)])):
        outs, lg = m4.forward(clean, pi)
        l_out, l_lg = loop_forward(shape, w, clean, pi=pi, codec=Rtn(4))
        assert _rel(lg, l_lg) < 1e-12, sorted(pi)
        for s, nm in snd.items():
            assert _rel(outs[s].reshape(l_out[nm].shape), l_out[nm]) < 1e-12, (sorted(pi), nm)
    _, full4 = m4.forward(clean, ALL)
    _, full8 = m8.forward(clean, ALL)
    assert np.array_equal(full4, full8)
    _, lg4 = m4.forward(clean, frozenset())
    _, lg8 = m8.forward(clean, frozenset())
    assert np.abs(lg4 - full8).max() > 3 * np.abs(lg8 - full8).max()
    with pytest.raises(ValueError):
        Model(shape, w, low_bits=12)
