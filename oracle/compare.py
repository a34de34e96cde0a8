"""Comparison rules between the HIP path and the oracle.  TEST INFRASTRUCTURE ONLY.

Integers (counts, ready ids, groupings) are compared bit for bit.  Floating-point tensors are
compared row by row in the max norm: a row passes when

    max_j |got[r, j] - ref[r, j]|  <=  rel * max(max_j |ref[r, j]|, 1e-3 * max |ref|)

with rel = 1e-5 for fp32 workloads and 2e-2 for bf16 workloads.  The floor keeps rows that
nearly cancel from demanding more than the arithmetic can give.  A row that is a sum (an average of
M gradients, a running sum) is measured against its largest term when the caller passes
`term_scale`: the rounding error of a sum is bounded by the size of its terms, not of its value,
and two gradients of opposite sign can cancel to a fraction of either.  Rows of views whose hidden
pre-activations sit within rounding distance of the ReLU kink may legitimately take the other
branch; callers pass them as `exempt` and they are only required to be finite.
"""
from __future__ import annotations

import numpy as np

REL = {"f32": 1e-5, "bf16": 2e-2}


def row_errors(got, ref, term_scale=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if got.ndim == 1:
        got, ref = got.reshape(1, -1), ref.reshape(1, -1)
    if ref.size == 0:
        return np.zeros(ref.shape[0]), np.ones(ref.shape[0])
    err = np.abs(got - ref).max(axis=1)
    scale = np.maximum(np.abs(ref).max(axis=1), 1e-3 * np.abs(ref).max())
    if term_scale is not None:
        scale = np.maximum(scale, np.asarray(term_scale, dtype=np.float64).reshape(-1))
    return err, scale


def assert_rows_close(got, ref, rel, what, exempt=None, term_scale=None):
    """Returns the worst err/scale ratio (for reporting)."""
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    err, scale = row_errors(got, ref, term_scale)
    ok = err <= rel * scale
    if exempt is not None:
        ok = ok | np.asarray(exempt, dtype=bool)
    if not ok.all():
        bad = np.flatnonzero(~ok)
        r = bad[np.argmax((err / np.maximum(scale, 1e-300))[bad])]
        raise AssertionError(f"{what}: {len(bad)} of {len(ok)} rows outside rel {rel:g}; worst row {r}: "
                             f"err {err[r]:.3e} vs scale {scale[r]:.3e} (ratio {err[r] / max(scale[r], 1e-300):.3e})")
    masked = np.where(np.asarray(exempt, dtype=bool), 0.0, err / np.maximum(scale, 1e-300)) if exempt is not None \
        else err / np.maximum(scale, 1e-300)
    return float(masked.max()) if masked.size else 0.0
