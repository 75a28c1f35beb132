"""bfloat16 storage helpers (numpy has no bfloat16 dtype).

A bfloat16 value is the upper 16 bits of an IEEE-754 binary32.  Inputs that a
bf16 configuration feeds to both the oracle and the GPU are rounded ONCE here
(round to nearest, ties to even) so both sides start from identical values.
"""
import numpy as np


def f32_to_bf16_bits(a):
    """float32 array -> uint16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r.reshape(a.shape)


def bf16_bits_to_f32(b):
    """uint16 bit patterns -> float32 values (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def bf16_round(a):
    """float array -> float32 array whose every value is bf16-representable."""
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))


def f16_round(a):
    """float array -> float32 array whose every value is representable in IEEE half precision
    (numpy's float16 conversion rounds to nearest, ties to even)."""
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)
