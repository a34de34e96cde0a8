"""Counter-based table initialiser of the oracle.  TEST INFRASTRUCTURE ONLY.

The step's tables are initialised with zero-mean noise of a given standard
deviation (Section 4.1 only says every variable starts from a fixed standard
deviation).  So that a 12.8 GB table never has to be copied between the two
sides, both derive element (row, col) of table `stream` from a counter-based
generator:

  * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
    easy as 1, 2, 3", SC'11) with counter (idx_lo, idx_hi, stream, 0) and key
    (seed_lo, seed_hi), idx = row * dim + col;
  * the four 32-bit outputs are cut into eight 16-bit halves whose sum S is an
    Irwin-Hall variate: (S - 4*65535) has mean 0 and variance 8*(65536^2-1)/12;
  * value = fp32(S - 4*65535) * fp32(std / sqrt(8*(65536^2-1)/12)), one fp32
    multiply, then rounded to the table's storage type.

Only integer arithmetic and one IEEE multiply are involved, so the result is a
fixed bit pattern per (seed, stream, row, col).
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32 on arrays of 32-bit counters (held in uint64)."""
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
    return c0, c1, c2, c3


def irwin_hall_scale(std: float) -> np.float32:
    var = 8.0 * (65536.0 * 65536.0 - 1.0) / 12.0
    return np.float32(np.float64(std) / np.sqrt(np.float64(var)))


def centred_sums(seed: int, stream: int, idx: np.ndarray) -> np.ndarray:
    """Integer Irwin-Hall variate (S - 4*65535) for flat element indices idx."""
    idx = np.asarray(idx, dtype=np.uint64)
    w = philox4x32_10(idx & _MASK, idx >> _S32, np.uint64(stream), np.uint64(0),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    s = np.zeros(idx.shape, dtype=np.int64)
    for word in w:
        s += (word & np.uint64(0xFFFF)).astype(np.int64)
        s += (word >> np.uint64(16)).astype(np.int64)
    return s - 4 * 65535


def normal_f32(seed: int, stream: int, idx: np.ndarray, std: float) -> np.ndarray:
    """fp32 values of the initialiser at flat indices idx."""
    s = centred_sums(seed, stream, idx).astype(np.float32)
    return s * irwin_hall_scale(std)


def normal_rows(seed: int, stream: int, row_ids, dim: int, std: float) -> np.ndarray:
    """[len(row_ids) x dim] fp32 block of table `stream`."""
    rows = np.asarray(row_ids, dtype=np.uint64).reshape(-1, 1)
    cols = np.arange(dim, dtype=np.uint64).reshape(1, -1)
    return normal_f32(seed, stream, rows * np.uint64(dim) + cols, std)
