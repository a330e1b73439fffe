"""Storage-format conversions for the oracle (test infrastructure; shares nothing with the HIP path).

bfloat16 = the upper 16 bits of an IEEE binary32 value (8 exponent bits, 7 stored
significand bits).  Arrays of bf16 values are carried as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to bf16 with a single round-to-nearest-even step (finite inputs).

    Going through float32 with two nearest roundings can land on the wrong side of
    a tie, so the first step is made 'round to odd': truncate to float32 toward
    zero and set the last bit if anything was lost.  Rounding that 24-bit value to
    8 bits, nearest-even, then equals rounding the original once.
    """
    x = np.ascontiguousarray(x, dtype=np.float64)
    f = x.astype(np.float32)
    too_big = np.abs(f.astype(np.float64)) > np.abs(x)
    f = np.where(too_big, np.nextafter(f, np.float32(0.0)), f).astype(np.float32)
    u = f.view(np.uint32).copy()
    inexact = f.astype(np.float64) != x
    u[inexact] |= np.uint32(1)
    keep_low = (u >> np.uint32(16)) & np.uint32(1)
    r = (u.astype(np.uint64) + np.uint64(0x7FFF) + keep_low.astype(np.uint64)) >> np.uint64(16)
    return r.astype(np.uint16)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Widen a stored tensor ('f32' float32 array or 'bf16' uint16 bit patterns) to float64, exactly."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(a)
    raise ValueError(dtype)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values once, to nearest-even, into the storage format."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        return f64_to_bf16_bits(x)
    raise ValueError(dtype)
