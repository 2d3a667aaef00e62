"""Integer round-to-nearest quantiser, Eq. RTN-Q as printed (test infrastructure).

Paper, Appendix "Quantization", Eq. RTN-Q:  Q(w) = step * Round(w / step),  step = max|w| / 2^(N-1),
N the number of bits; used here for the 4-bit point of the bit-width ablation (Sec. "Ablation Studies",
Different Quantization Precisions).  The grid is the integer multiples of the step; the largest magnitude
of the group lands on the multiple 2^(N-1) exactly (so a group uses the 2^N + 1 multiples -2^(N-1) ..
2^(N-1): the formula as printed, not a two's-complement range).

Readings where the paper is silent: Round is round-half-to-even; one group per weight slice and per
activation row, the groups of the 8-bit quantiser (e4m3.py).  As there, every operation is a single IEEE
binary32 operation so that a device reproduces multiples and steps bit for bit:

    amax = max |x|                       (exact)
    step = amax / 2^(N-1)                (exact: a power of two; step = 1 when amax = 0)
    inv  = 1 / step                      (binary32 division)
    k    = nearest-even integer of x * inv   (binary32 product)

The interface is that of e4m3.py -- quantize_groups, quantize_rows, decode -- with the integer multiple
in the place of the code.

parity unpinned: none -- tests/test_oracle_rtn.py holds it to Python's own integer rounding of exact
fractions, to the closed forms of the grid and to the half-step error bound.
"""
import numpy as np


class Rtn:
    def __init__(self, bits):
        if not 2 <= bits <= 8:
            raise ValueError("bits")
        self.bits = bits
        self.top = np.float32(2.0 ** (bits - 1))

    def quantize_groups(self, x, axis=-1):
        """(multiples int16 like x, steps float32 with `axis` reduced; axis None = one group)."""
        x = np.asarray(x, dtype=np.float32)
        if np.isnan(x).any():
            raise ValueError("NaN entering the quantiser")
        if axis is None:
            amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0)
            step = np.float32(1.0) if amax == 0 else np.float32(amax / self.top)
            inv = np.float32(np.float32(1.0) / step)
            return np.rint(x * inv).astype(np.int16), step
        amax = np.max(np.abs(x), axis=axis, keepdims=True).astype(np.float32)
        step = np.where(amax == 0, np.float32(1.0), amax / self.top).astype(np.float32)
        inv = (np.float32(1.0) / step).astype(np.float32)
        y = (x * inv).astype(np.float32)
        return np.rint(y).astype(np.int16), np.squeeze(step, axis=axis)

    def quantize_rows(self, x):
        return self.quantize_groups(x, axis=-1)

    @staticmethod
    def decode(k):
        return np.asarray(k).astype(np.float64)
