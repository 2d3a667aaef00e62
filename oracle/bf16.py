"""bfloat16 rounding as a quantiser (test infrastructure).

Paper, Sec. "Selective Precision Allocation Strategy": the components that are not attention heads run in
bfloat16.  bfloat16 is binary32 cut to 1 sign, 8 exponent and 7 stored mantissa bits; a value is rounded to
the nearest such number, ties to the even mantissa.  There is no scale: the format keeps binary32's range.

The interface is that of e4m3.py -- quantize_groups, quantize_rows, decode -- with the 16-bit pattern as the
code and a scale of one, so that the model code treats the three grids alike.  x is rounded to binary32 first
(a no-op for binary32 input): a device holds binary32 values at this point.

parity unpinned: none -- tests/test_oracle_bf16.py holds encode / decode to the closed form of the format, to
exhaustive nearest-neighbour search on a binade, to ties, and to torch's own conversion.
"""
import numpy as np


def encode(x):
    """Nearest-even bfloat16 bit pattern (uint16) of each binary32 value."""
    x = np.asarray(x, dtype=np.float32)
    if not np.isfinite(x).all():
        raise ValueError("non-finite value entering the bfloat16 rounding")
    u = x.view(np.uint32).astype(np.uint64)
    keep = u >> np.uint64(16)                      # the bits bfloat16 keeps
    rest = u & np.uint64(0xFFFF)                   # the 16 mantissa bits it drops
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint64(1)) == 1))
    code = (keep + up.astype(np.uint64)).astype(np.uint32)
    if ((code & 0x7F80) == 0x7F80).any():
        raise ValueError("value rounds to infinity in bfloat16")
    return code.astype(np.uint16)


def decode(codes):
    """float64 value of each bfloat16 bit pattern."""
    c = np.asarray(codes, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return c.view(np.float32).astype(np.float64)


def quantize_groups(x, axis=-1):
    x = np.asarray(x, dtype=np.float32)
    codes = encode(x)
    if axis is None:
        return codes, np.float32(1.0)
    shape = list(x.shape)
    del shape[axis]
    return codes, np.ones(shape, dtype=np.float32)


def quantize_rows(x):
    return quantize_groups(x, axis=-1)
