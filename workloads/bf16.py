"""bfloat16 <-> float32 bit conversion in NumPy (storage format only).

bf16 is the upper 16 bits of an IEEE-754 binary32 value.  Rounding from fp32
is round-to-nearest, ties-to-even, done once when a workload is generated so
that every consumer sees the same bits.
"""
import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest-even) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # add 0x7FFF plus the lowest kept bit: classic nearest-even on truncation
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Expand uint16 bf16 bit patterns to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
