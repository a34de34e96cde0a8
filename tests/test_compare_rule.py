"""The comparison rule that the GPU parity tests rely on, checked on hand-made rows: a comparator that
quietly accepted more than it states would make every parity test weaker without turning one red."""
import numpy as np
import pytest

from oracle.compare import REL, assert_delta_rows_close, assert_rows_close, row_errors, ulp


def test_tolerances_are_the_stated_ones():
    assert REL == {"f32": 1e-5, "bf16": 2e-2}


def test_units_in_the_last_place():
    assert ulp(1.0, "f32") == 2.0 ** -23 and ulp(1.999, "f32") == 2.0 ** -23 and ulp(2.0, "f32") == 2.0 ** -22
    assert ulp(1.5, "bf16") == 2.0 ** -7 and ulp(-3.0, "bf16") == 2.0 ** -6 and ulp(0.01, "bf16") == 2.0 ** -14
    assert ulp(0.0, "f32") == 2.0 ** (-126 - 23)
    assert np.array_equal(ulp(np.array([1.0, 4.0]), "f64"), [2.0 ** -52, 2.0 ** -50])


def test_a_row_is_measured_against_its_own_largest_element():
    ref = np.array([[1.0, 0.5, 0.0], [100.0, 0.0, 0.0]])
    good = ref + np.array([[0.9e-5, 0, 0], [0, 0.9e-3, 0]])
    assert_rows_close(good, ref, 1e-5, "rows")
    # the same absolute error that row 1 may have is too much for row 0 ...
    with pytest.raises(AssertionError, match="1 of 2 rows"):
        assert_rows_close(ref + np.array([[0, 0.9e-3, 0], [0, 0, 0]]), ref, 1e-5, "rows")
    # ... and just over the bar fails, in any column
    with pytest.raises(AssertionError):
        assert_rows_close(ref + np.array([[0, 0, 1.1e-5], [0, 0, 0]]), ref, 1e-5, "rows")
    with pytest.raises(AssertionError, match="non-finite"):
        assert_rows_close(ref * np.array([[1.0], [np.nan]]), ref, 1e-5, "rows")
    with pytest.raises(AssertionError):
        assert_rows_close(ref[:, :2], ref, 1e-5, "rows")


def test_the_floor_is_a_thousandth_of_the_largest_element_of_the_tensor():
    ref = np.array([[1000.0, 0.0], [1e-6, 0.0]])
    err, scale = row_errors(ref, ref)
    assert scale.tolist() == [1000.0, 1.0] and err.tolist() == [0.0, 0.0]
    assert_rows_close(ref + np.array([[0, 0], [0, 0.9e-5]]), ref, 1e-5, "floor")
    with pytest.raises(AssertionError):
        assert_rows_close(ref + np.array([[0, 0], [0, 1.1e-5]]), ref, 1e-5, "floor")


def test_a_sum_is_measured_against_its_largest_term_when_given():
    ref = np.array([[1e-3, 0.0], [1.0, 0.0]])                # row 0: two terms of size 5 that nearly cancel
    got = ref + np.array([[4e-5, 0], [0, 0]])
    with pytest.raises(AssertionError):
        assert_rows_close(got, ref, 1e-5, "sum")
    assert_rows_close(got, ref, 1e-5, "sum", term_scale=[5.0, 0.0])
    with pytest.raises(AssertionError):
        assert_rows_close(ref + np.array([[6e-5, 0], [0, 0]]), ref, 1e-5, "sum", term_scale=[5.0, 0.0])


def test_exempt_rows_are_held_to_their_bound_and_other_rows_to_the_rule():
    ref = np.ones((3, 2))
    got = ref + np.array([[0.05, 0], [0, 0], [0, 0]])
    with pytest.raises(AssertionError, match="need a bound"):
        assert_rows_close(got, ref, 1e-5, "exempt", exempt=[True, False, False])
    assert assert_rows_close(got, ref, 1e-5, "exempt", exempt=[True, False, False], exempt_bound=[0.1, 0, 0]) == 0.0
    with pytest.raises(AssertionError):                      # beyond its bound
        assert_rows_close(got, ref, 1e-5, "exempt", exempt=[True, False, False], exempt_bound=[0.04, 0, 0])
    with pytest.raises(AssertionError):                      # the bound of an exempt row does not cover another row
        assert_rows_close(got, ref, 1e-5, "exempt", exempt=[False, True, False], exempt_bound=[0.1, 0.1, 0.1])


def test_updates_are_compared_as_changes():
    before = np.array([[1.0, 2.0], [3.0, 4.0]])
    change = np.array([[1e-4, -2e-4], [0.0, 3e-4]])
    ref_after = before + change
    # the same change on the other side, off by less than rel of the change plus one storage ulp
    got_after = before + change * (1 + 0.5e-5)
    worst, resolution = assert_delta_rows_close(got_after, before, ref_after, before, 1e-5, "f64", 1, "delta")
    assert worst < 1.0 and resolution > 1e4
    # an update that did not happen is far outside, although after-vs-after it would be within 1e-3 relative
    with pytest.raises(AssertionError, match="change of 2 of 2 rows"):
        assert_delta_rows_close(before, before, ref_after, before, 1e-5, "f64", 1, "delta")
    # half the change, the wrong sign, the change applied to the wrong row: all outside
    for wrong in (before + 0.5 * change, before - change, before + change[::-1]):
        with pytest.raises(AssertionError):
            assert_delta_rows_close(wrong, before, ref_after, before, 1e-5, "f64", 1, "delta")
    # one rounding of the new value into the storage type is allowed per step, and no more
    one_ulp = ulp(4.0, "f32")
    assert_delta_rows_close(ref_after + np.array([[0, 0], [0, 0.9 * one_ulp]]), before, ref_after, before, 0.0, "f32", 1, "ulp")
    with pytest.raises(AssertionError):
        assert_delta_rows_close(ref_after + np.array([[0, 0], [0, 1.1 * one_ulp]]), before, ref_after, before, 0.0, "f32", 1, "ulp")
    assert_delta_rows_close(ref_after + np.array([[0, 0], [0, 2.9 * one_ulp]]), before, ref_after, before, 0.0, "f32", 3, "ulp")
    # a change below the resolution of the comparison says so in what it returns
    tiny_after = before + 1e-9
    _, resolution = assert_delta_rows_close(tiny_after, before, tiny_after, before, 1e-5, "f32", 1, "tiny")
    assert resolution < 1.0
