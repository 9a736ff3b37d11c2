"""bf16 <-> fp64 conversions for the oracle (own implementation).

bf16 = 1 sign, 8 exponent, 7 mantissa bits (the top half of an IEEE fp32).
Rounding is to nearest, ties to even, done directly from fp64 so that there
is no double rounding through fp32.
"""
from __future__ import annotations

import numpy as np

_MIN_NORMAL = 2.0 ** -126
_SUB_STEP = 2.0 ** -133          # spacing of bf16 subnormals
_MAX_FINITE = (2.0 - 2.0 ** -7) * 2.0 ** 127


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> exact fp64 values."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_f64(x: np.ndarray) -> np.ndarray:
    """fp64 -> nearest bf16-representable fp64 (ties to even)."""
    x = np.asarray(x, dtype=np.float64)
    u = x.view(np.uint64) if x.flags["C_CONTIGUOUS"] else np.ascontiguousarray(x).view(np.uint64)
    # keep 7 of the 52 mantissa bits: drop 45, round half to even on the kept lsb
    lsb = (u >> np.uint64(45)) & np.uint64(1)
    r = (u + np.uint64((1 << 44) - 1) + lsb) & ~np.uint64((1 << 45) - 1)
    y = r.view(np.float64).copy()
    small = np.abs(x) < _MIN_NORMAL
    if small.any():
        y[small] = np.round(x[small] / _SUB_STEP) * _SUB_STEP
    big = np.abs(y) > _MAX_FINITE
    if big.any():
        y[big] = np.sign(y[big]) * np.inf
    return y.reshape(x.shape)


def f64_to_bits(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bit patterns (uint16), rounding to nearest even."""
    y = round_f64(x).astype(np.float32)      # exact: y is bf16-representable
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
