"""Precision helper: the one low-precision rounding the oracle imitates."""
import numpy as np


def round_to_bf16(x):
    """Round fp32 values to bfloat16 with round-to-nearest-even and return them
    as float64.  bf16 is the upper 16 bits of an IEEE fp32; rounding adds
    0x7FFF plus the lowest kept bit before truncating (finite inputs only)."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = ((bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = rounded.astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(x))
