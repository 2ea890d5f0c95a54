"""Storage rounding used when the device path keeps activations in a narrower type (oracle side; test
infrastructure). The paper has no reduced precision; the bf16 configuration is this repository's, and its
oracle is the fp64 computation with values rounded where the device stores them.

bf16 = the upper 16 bits of an IEEE binary32: 1 sign, 8 exponent, 7 fraction bits; conversion rounds to
nearest, ties to the even fraction. NaN and infinities keep their class.
"""
from __future__ import annotations

import numpy as np


def round_bf16(a) -> np.ndarray:
    """Nearest bf16 value (ties to even) of every element, returned as float64."""
    f32 = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f32.view(np.uint32).astype(np.uint64)
    lower = bits & 0xFFFF                       # the 16 bits that are dropped
    upper = bits >> 16
    half = 0x8000
    round_up = (lower > half) | ((lower == half) & ((upper & 1) == 1))
    upper = upper + round_up.astype(np.uint64)  # a carry into the exponent is the correct next binade / infinity
    out = (upper << 16).astype(np.uint32).view(np.float32)
    nan = np.isnan(f32)
    if nan.any():
        out = np.where(nan, np.float32(np.nan), out)
    return out.astype(np.float64).reshape(np.shape(a))


def round_f32(a) -> np.ndarray:
    """Nearest binary32 value of every element, returned as float64."""
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
