"""Distance in units in the last place between two arrays of bit patterns."""
from __future__ import annotations

import numpy as np


def ordered(bits: np.ndarray) -> np.ndarray:
    """Map sign-magnitude float bit patterns (uint16 or float32) to integers
    whose order is the order of the values; +0 and -0 both map to 0."""
    if bits.dtype == np.float32:
        u = bits.view(np.uint32).astype(np.int64)
        signbit = 1 << 31
    elif bits.dtype == np.uint16:
        u = bits.astype(np.int64)
        signbit = 1 << 15
    else:
        raise TypeError(bits.dtype)
    mag = u & (signbit - 1)
    return np.where(u & signbit, -mag, mag)


def ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    return np.abs(ordered(a) - ordered(b))
