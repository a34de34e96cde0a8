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
branch; callers pass them as `exempt` together with `exempt_bound`, the multiple of the row's scale
such a row may be off by at most.

What a step *changes* (table rows, MLP parameters) is compared as a change: after - before on both
sides, by the same row rule on the scale of the change, plus one unit in the last place of the
storage type per step, because either side rounds the new value into that type once per step.
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


_FRACTION_BITS = {"f32": 23, "bf16": 7, "f64": 52}


def ulp(magnitude, dtype: str):
    """Spacing of `dtype` numbers at |magnitude| (normal range)."""
    m = np.maximum(np.abs(np.asarray(magnitude, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(m)) - _FRACTION_BITS[dtype])


def assert_delta_rows_close(got_after, got_before, ref_after, ref_before, rel, storage, steps, what, term_scale=None):
    """The change of each row against the change of its reference; returns (worst ratio of the error to
    its allowance, smallest ratio of a reference row's change to its allowance): the second says how far
    above the resolution of the comparison the changes are (a step that changed nothing fails when it
    is well above 1)."""
    ga, gb = np.asarray(got_after, dtype=np.float64), np.asarray(got_before, dtype=np.float64)
    ra, rb = np.asarray(ref_after, dtype=np.float64), np.asarray(ref_before, dtype=np.float64)
    assert ga.shape == gb.shape == ra.shape == rb.shape, (ga.shape, gb.shape, ra.shape, rb.shape)
    assert np.all(np.isfinite(ga)), f"{what}: non-finite values"
    if ga.ndim == 1:
        ga, gb, ra, rb = (a.reshape(1, -1) for a in (ga, gb, ra, rb))
    if ra.size == 0:
        return 0.0, np.inf
    err, scale = row_errors(ga - gb, ra - rb, term_scale)
    allow = rel * scale + steps * ulp(np.maximum(np.abs(ra), np.abs(rb)).max(axis=1), storage)
    bad = np.flatnonzero(err > allow)
    if len(bad):
        r = bad[np.argmax(err[bad] / allow[bad])]
        raise AssertionError(f"{what}: change of {len(bad)} of {len(err)} rows outside rel {rel:g}; worst row {r}: "
                             f"err {err[r]:.3e}, change {np.abs(ra - rb)[r].max():.3e}, allowed {allow[r]:.3e}")
    return float((err / allow).max()), float(np.median(np.abs(ra - rb).max(axis=1) / allow))


def assert_rows_close(got, ref, rel, what, exempt=None, term_scale=None, exempt_bound=None):
    """Returns the worst err/scale ratio (for reporting)."""
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    err, scale = row_errors(got, ref, term_scale)
    ok = err <= rel * scale
    if exempt is not None:
        assert exempt_bound is not None, "exempt rows need a bound"
        ok = ok | (np.asarray(exempt, dtype=bool) & (err <= np.asarray(exempt_bound, dtype=np.float64) * scale))
    if not ok.all():
        bad = np.flatnonzero(~ok)
        r = bad[np.argmax((err / np.maximum(scale, 1e-300))[bad])]
        raise AssertionError(f"{what}: {len(bad)} of {len(ok)} rows outside rel {rel:g}; worst row {r}: "
                             f"err {err[r]:.3e} vs scale {scale[r]:.3e} (ratio {err[r] / max(scale[r], 1e-300):.3e})")
    masked = np.where(np.asarray(exempt, dtype=bool), 0.0, err / np.maximum(scale, 1e-300)) if exempt is not None \
        else err / np.maximum(scale, 1e-300)
    return float(masked.max()) if masked.size else 0.0
