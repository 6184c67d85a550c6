"""bf16 <-> float conversions (round-to-nearest-even), numpy only."""
import numpy as np


def bf16_bits(x):
    """Round float values to bf16 (nearest, ties to even); return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b):
    """Widen 16-bit bf16 patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x):
    """Round to bf16 and widen again: a float32 array of bf16-representable values."""
    return bf16_from_bits(bf16_bits(x))
