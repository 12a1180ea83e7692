"""bfloat16 storage format for the oracle (test infrastructure).

bfloat16 is the upper 16 bits of an IEEE-754 binary32.  The KV cache stores
bfloat16, so the oracle rounds exactly once, at the cache write, with
round-to-nearest, ties-to-even.  Values travel as uint16 bit patterns because
numpy has no bfloat16 dtype.
"""
import numpy as np


def to_bits(x):
    """float32 array -> uint16 bfloat16 bit patterns (round-to-nearest-even).

    NaN stays NaN (quiet bit forced); +-inf and overflow behave as IEEE RNE.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1                       # last kept bit: decides ties
    rounded = (u + 0x7FFF + lsb) >> 16
    is_nan = (u & 0x7FFFFFFF) > 0x7F800000
    rounded = np.where(is_nan, (u >> 16) | 0x40, rounded)
    return (rounded & 0xFFFF).astype(np.uint16)


def from_bits(b, dtype=np.float32):
    """uint16 bfloat16 bit patterns -> float array of the same values (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    f = (b.astype(np.uint32) << 16).view(np.float32)
    return f.astype(dtype, copy=False)


def round_trip(x):
    """float32 array -> the float32 values bfloat16 storage would hold."""
    return from_bits(to_bits(x))
