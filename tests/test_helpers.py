"""The closeness criteria of the parity tests must see what a whole-tensor norm hides: one wrong row of an
activation, one wrong element of a parameter tensor.  CPU only: the mistakes are planted in host copies."""
import numpy as np
import pytest

from helpers import MAX_ABS_FACTOR, assert_close, closeness, max_abs_ratio, rel_l2, worst_row_rel_l2

RNG = np.random.default_rng(7)
TOL = 2e-2


def _activation(rows=8320, dim=384):
    ref = RNG.standard_normal((rows, dim))
    got = ref * (1.0 + 2e-3 * RNG.standard_normal(ref.shape))      # an honest low-precision result
    return got, ref


def test_an_honest_result_passes_all_three_criteria():
    got, ref = _activation()
    c = assert_close(got, ref, TOL, "x_out", row_len=384)
    assert c["rel_l2"] < 3e-3 and c["row"] < 4e-3 and c["max_abs"] < 8e-3   # multiplicative errors peak at the largest values: about 3x the norm ratio


def test_one_wrong_row_among_thousands_passes_the_norm_and_fails_the_row_criterion():
    got, ref = _activation()
    got[4711] = got[12]                                             # a row written to the wrong place
    assert rel_l2(got, ref) < TOL                                   # the whole-tensor norm does not see it
    assert worst_row_rel_l2(got, ref, 384) > 1.0
    with pytest.raises(AssertionError, match="worst row"):
        assert_close(got, ref, 0.5, "x_out", row_len=384, row_tol=TOL)   # even with the other criteria wide open
    with pytest.raises(AssertionError):
        assert_close(got, ref, TOL, "x_out", row_len=384)


def test_one_wrong_element_of_a_weight_gradient_fails_the_element_criterion():
    ref = 0.02 * RNG.standard_normal((384, 1536))
    got = ref * (1.0 + 2e-3 * RNG.standard_normal(ref.shape))
    i = np.unravel_index(np.argsort(np.abs(ref), axis=None)[ref.size // 2], ref.shape)   # an element of median size
    got[i] = -got[i]                                                # sign error in a single element
    assert rel_l2(got, ref) < TOL
    assert max_abs_ratio(got, ref) > MAX_ABS_FACTOR * TOL
    with pytest.raises(AssertionError, match="largest element error"):
        assert_close(got, ref, TOL, "fc1.w gradient")


def test_one_dropped_bias_element_fails():
    ref = 0.5 + 0.1 * RNG.standard_normal(1536)
    got = ref.copy()
    got[100] = 0.0                                                  # an element nobody wrote
    with pytest.raises(AssertionError):
        assert_close(got, ref, TOL, "fc1.b")
    got = ref.copy()
    got[7] = np.nan
    with pytest.raises(AssertionError, match="non-finite"):
        assert_close(got, ref, TOL, "fc1.b")


def test_rows_emptied_by_a_relu_are_measured_on_the_tensors_own_scale():
    ref = np.maximum(RNG.standard_normal((1000, 32)), 0.0)
    ref[::7] = 0.0                                                  # pixels with every channel switched off
    got = ref + 1e-3 * RNG.standard_normal(ref.shape)
    c = closeness(got, ref, row_len=32)
    assert c["row"] < 5e-3                                          # not divided by a zero row norm
    got[14] = 1.0                                                   # an empty row that came back full
    assert worst_row_rel_l2(got, ref, 32) > 1.0


def test_reference_of_zeros_is_compared_absolutely():
    assert rel_l2(np.full(5, 1e-3), np.zeros(5)) == pytest.approx(np.sqrt(5) * 1e-3)
    assert max_abs_ratio(np.full(5, 1e-3), np.zeros(5)) == pytest.approx(1e-3)
