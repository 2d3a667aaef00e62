"""FP8 E4M3 codec and the round-to-nearest quantiser (test infrastructure).

Format (paper, Sec. "Direct Quantization Does Not Work on ACDC", footnote on
FP8_E4M3; Appendix "Environment"): 1 sign, 4 exponent, 3 mantissa bits, with a
smallest normal step of 2^-6.  That fixes the exponent bias at 7, i.e. the
OCP "E4M3FN" encoding:

    normal     (-1)^s * 2^(e-7) * (1 + m/8)      e = 1..15
    subnormal  (-1)^s * 2^-6    * (m/8)          e = 0
    max finite 448 (e=15, m=6);  e=15, m=7 is NaN;  no infinities.

Quantiser (paper, Appendix "Quantization", Eq. RTN-Q, re-read for a float
grid): the scale is fixed by the absolute maximum of the group so that it
maps to the top of the grid (448); values are rounded to the nearest grid
point, ties to the even mantissa.  Every operation of the quantiser is a
single IEEE binary32 operation so a device can reproduce codes and scales
bit for bit:

    amax  = max |x|                      (exact)
    scale = amax / 448     (binary32 division; scale = 1 when amax = 0)
    inv   = 1 / scale      (binary32 division)
    y     = x * inv        (binary32 multiplication)
    code  = nearest-even e4m3(y), |y| > 448 saturates to +-448, sign kept for -0

parity unpinned: none -- decode is pinned by the closed form above over all
256 codes, encode by round trips, midpoints and the saturation cases.
"""
import numpy as np

E4M3_MAX = np.float32(448.0)


def decode_table():
    """float64[256]: value of each code (NaN for 0x7F and 0xFF)."""
    t = np.empty(256, dtype=np.float64)
    for c in range(256):
        s = -1.0 if c & 0x80 else 1.0
        e = (c >> 3) & 0xF
        m = c & 7
        if e == 15 and m == 7:
            t[c] = np.nan
        elif e == 0:
            t[c] = s * 2.0 ** -6 * (m / 8.0)
        else:
            t[c] = s * 2.0 ** (e - 7) * (1.0 + m / 8.0)
    return t


_DEC = decode_table()
# positive finite grid, ascending: codes 0x00..0x7E
_GRID = _DEC[:0x7F].copy()


def decode(codes):
    return _DEC[np.asarray(codes, dtype=np.uint8)]


def encode(y):
    """Nearest-even e4m3 code of each binary32 value in y (saturating).

    Written as a search over the 127-point positive grid so that it is
    obviously the definition: pick the nearest grid point; on an exact tie
    pick the one whose code is even (its mantissa LSB is 0).
    """
    y = np.asarray(y, dtype=np.float32)
    if np.isnan(y).any():
        raise ValueError("NaN entering the e4m3 encoder")
    a = np.abs(y).astype(np.float64)
    a = np.minimum(a, 448.0)
    hi = np.searchsorted(_GRID, a, side="left")          # first grid index with grid >= a
    hi = np.minimum(hi, 0x7E)
    lo = np.maximum(hi - 1, 0)
    dlo = a - _GRID[lo]
    dhi = _GRID[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((hi & 1) == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    sign = np.signbit(y).astype(np.uint8) << 7
    return (code | sign).astype(np.uint8)


def quantize_groups(x, axis=-1):
    """Quantise x with one scale per slice along `axis` (None = one scale for all of x).

    Returns (codes uint8 like x, scales float32 with `axis` reduced).
    x is rounded to binary32 first (a no-op for binary32 input).
    """
    x = np.asarray(x, dtype=np.float32)
    if axis is None:
        amax = np.max(np.abs(x)) if x.size else np.float32(0)
        amax = np.float32(amax)
        scale = np.float32(1.0) if amax == 0 else np.float32(amax / E4M3_MAX)
        inv = np.float32(np.float32(1.0) / scale)
        y = x * inv
        return encode(y), scale
    amax = np.max(np.abs(x), axis=axis, keepdims=True).astype(np.float32)
    scale = np.where(amax == 0, np.float32(1.0), amax / E4M3_MAX).astype(np.float32)
    inv = (np.float32(1.0) / scale).astype(np.float32)
    y = (x * inv).astype(np.float32)
    return encode(y), np.squeeze(scale, axis=axis)


def quantize_rows(x):
    """One scale per row (last axis) -- the activation quantiser."""
    return quantize_groups(x, axis=-1)


def dequantize(codes, scale, axis=-1):
    s = np.asarray(scale, dtype=np.float64)
    if axis is not None and s.ndim:
        s = np.expand_dims(s, axis)
    return decode(codes) * s
