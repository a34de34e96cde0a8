"""Storage roundings applied by the oracle.  TEST INFRASTRUCTURE ONLY.

The oracle computes in fp64.  Where a workload stores a tensor in fp32 or
bfloat16 the stored value is the fp64 result rounded once, to nearest with
ties to even, into that format.  bfloat16 = sign, 8 exponent bits (as fp32),
7 fraction bits.
"""
from __future__ import annotations

import numpy as np

_DROP = 45                      # fp64 has 52 fraction bits, bfloat16 keeps 7
_MIN_NORMAL = 2.0 ** -126       # smallest normal bfloat16 (same exponent range as fp32)
_SUB_QUANTUM = 2.0 ** -133      # spacing of bfloat16 subnormals
_OVERFLOW = 2.0 ** 128


def round_bf16(x) -> np.ndarray:
    """fp64 -> nearest bfloat16 (ties to even), returned as fp64."""
    x = np.array(x, dtype=np.float64, copy=True)
    flat = x.reshape(-1)
    bits = flat.view(np.uint64)
    mag = np.abs(flat)
    normal = (mag >= _MIN_NORMAL) & np.isfinite(flat)
    small = mag < _MIN_NORMAL

    lsb = (bits >> np.uint64(_DROP)) & np.uint64(1)
    rounded = (bits + np.uint64((1 << (_DROP - 1)) - 1) + lsb) & ~np.uint64((1 << _DROP) - 1)
    out = np.where(normal, rounded, bits).view(np.float64)
    # gradual underflow: multiples of 2^-133, ties to even (rint), sign kept
    sub = np.rint(flat / _SUB_QUANTUM) * _SUB_QUANTUM
    out = np.where(small, np.copysign(sub, flat), out)
    out = np.where(np.abs(out) >= _OVERFLOW, np.copysign(np.inf, out), out)
    out = np.where(np.isnan(flat), np.nan, out)
    return out.reshape(x.shape)


def round_f32(x) -> np.ndarray:
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_to(x, dtype: str) -> np.ndarray:
    """dtype in {"f64", "f32", "bf16"}."""
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return round_f32(x)
    if dtype == "bf16":
        return round_bf16(x)
    raise ValueError(f"unknown dtype {dtype!r}")
