"""The error metrics of the parity tests, tested on planted damage (CPU only): the per-row bound
must see what the whole-tensor norm cannot."""
import numpy as np
import pytest

from tests import parity_utils as U


def _pair(seed=0, tokens=8192, heads=4, d=128, noise=2e-3):
    rng = np.random.default_rng(seed)
    ref = rng.standard_normal((tokens, heads, d))
    return ref, ref * (1.0 + noise * rng.standard_normal(ref.shape))


def test_healthy_tensor_passes_both_bounds():
    ref, got = _pair()
    assert U.rel_rms(got, ref) <= U.TOL_GRAD_RELRMS
    assert U.assert_rows_close("dq", got, ref, U.TOL_GRAD_RELRMS) < 0.2


def test_one_unwritten_row_passes_the_tensor_norm_and_fails_the_row_bound():
    ref, got = _pair()
    got[100, 2] = 0.0
    assert U.rel_rms(got, ref) <= U.TOL_GRAD_RELRMS          # 1/sqrt(32768) = 5.5e-3: invisible
    with pytest.raises(AssertionError, match="row"):
        U.assert_rows_close("dq", got, ref, U.TOL_GRAD_RELRMS)


def test_one_wrong_four_element_chunk_fails_the_row_bound():
    ref, got = _pair(tokens=512, heads=2)
    got[7, 1, 4:8] = 0.0
    assert U.rel_rms(got, ref) <= U.TOL_GRAD_RELRMS
    with pytest.raises(AssertionError):
        U.assert_rows_close("dk", got, ref, U.TOL_GRAD_RELRMS)


def test_rows_small_by_cancellation_are_held_to_the_floor_not_to_themselves():
    ref, got = _pair()
    ref[5, 0] = 0.0
    got[5, 0] = 1e-6 * np.ones(128)                  # exact zero expected, rounding noise found
    U.assert_rows_close("dq", got, ref, U.TOL_GRAD_RELRMS)
    got[5, 0] = 1e-3 * np.ones(128)                  # a real error on a row that should be zero
    with pytest.raises(AssertionError):
        U.assert_rows_close("dq", got, ref, U.TOL_GRAD_RELRMS)


def test_nan_rows_fail():
    ref, got = _pair(tokens=64, heads=1)
    got[3, 0, 0] = np.nan
    with pytest.raises(AssertionError):
        U.assert_rows_close("out", got, ref, U.TOL_OUT_RELRMS)
