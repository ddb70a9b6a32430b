"""Pins of the error measures every parity test gates on (oracle/metrics.py).

Every expected value below is worked out by hand from the definitions
  M1 = max_i |got_i - ref_i| / ref_abs_i            (ref_abs = the contraction of absolute values)
  M2 = max_i |got_i - ref_i| / max(|ref_i|, rms(ref)),  rms(ref) = sqrt(mean(ref^2))
and written as a literal, so a slip in a denominator, a mean taken as a sum, a max taken as a min
or a dropped absolute value fails at least one case.
"""
import numpy as np
import pytest

from oracle.metrics import m1, m2, rel_l2


def test_m2_where_the_element_magnitude_is_the_denominator():
    # ref = [3, -4]: rms = sqrt((9 + 16) / 2) = 3.5355...; |ref_1| = 4 > rms, |ref_0| = 3 < rms.
    # errors: 0 and 0.4  ->  0.4 / 4 = 0.1
    assert m2([3.0, -3.6], [3.0, -4.0]) == pytest.approx(0.1, rel=1e-15)


def test_m2_where_rms_wins_over_a_small_element():
    # ref = [0.001, 1, -1, 1]: rms = sqrt((1e-6 + 3) / 4) = 0.8660255...
    # the only error sits on the small element: |0.101 - 0.001| = 0.1 -> 0.1 / rms (not 0.1 / 0.001 = 100)
    rms = np.sqrt((1e-6 + 3.0) / 4.0)
    got = m2([0.101, 1.0, -1.0, 1.0], [0.001, 1.0, -1.0, 1.0])
    assert got == pytest.approx(0.1 / rms, rel=1e-14)
    assert got == pytest.approx(0.11547, rel=1e-4)                      # the literal, for the eye


def test_m2_with_a_zero_reference_element_uses_rms():
    # ref = [0, 2]: rms = sqrt(4 / 2) = sqrt(2); error 0.5 on the zero element -> 0.5 / sqrt(2)
    assert m2([0.5, 2.0], [0.0, 2.0]) == pytest.approx(0.35355339059327373, rel=1e-15)


def test_m2_takes_the_maximum_over_elements_and_the_absolute_error():
    # ref = [10, 10, 10, 10] (rms 10): errors -1, +2, 0, -3  ->  0.3
    assert m2([9.0, 12.0, 10.0, 7.0], [10.0] * 4) == pytest.approx(0.3, rel=1e-15)
    # the sign of the error does not matter
    assert m2([11.0, 8.0, 10.0, 13.0], [10.0] * 4) == pytest.approx(0.3, rel=1e-15)


def test_m2_all_zero_reference_and_empty_input():
    assert m2([0.0, 0.0], [0.0, 0.0]) == 0.0
    assert m2([0.25, 0.0], [0.0, 0.0]) == 0.25                           # denominator falls back to 1
    assert m2(np.zeros((0, 3)), np.zeros((0, 3))) == 0.0


def test_m2_of_identical_arrays_is_zero_and_shape_is_irrelevant():
    ref = np.arange(24, dtype=np.float64).reshape(2, 3, 4) - 7.0
    assert m2(ref.copy(), ref) == 0.0
    got = ref.copy()
    got[1, 2, 3] += 1.6                                                  # ref there = 16, the largest: 0.1
    assert m2(got, ref) == pytest.approx(0.1, rel=1e-15)
    assert m2(got.reshape(-1), ref.reshape(-1)) == pytest.approx(0.1, rel=1e-15)


def test_m1_is_relative_to_the_contraction_of_absolute_values():
    # dot products x.y with cancellation: ref = [1 - 1, 2 + 2] = [0, 4], ref_abs = [2, 4]
    # got = [0.002, 4.002]  ->  max(0.002 / 2, 0.002 / 4) = 0.001
    assert m1([0.002, 4.002], [0.0, 4.0], [2.0, 4.0]) == pytest.approx(1e-3, rel=1e-12)
    # the larger error on the larger denominator: max(0.002 / 2, 0.02 / 4) = 0.005
    assert m1([0.002, 4.02], [0.0, 4.0], [2.0, 4.0]) == pytest.approx(5e-3, rel=1e-12)


def test_m1_zero_denominator_and_empty_input():
    # an output none of whose products is non-zero: the absolute error itself
    assert m1([0.5, 1.0], [0.0, 1.0], [0.0, 1.0]) == 0.5
    assert m1(np.zeros(0), np.zeros(0), np.zeros(0)) == 0.0


def test_m1_matches_the_textbook_bound_on_a_float32_dot_product():
    # fp32 accumulation of K products obeys |fl(x.y) - x.y| <= K * 2^-24 * |x|.|y| (to first order);
    # the measure of an honest fp32 dot product must sit below that and above zero
    rng = np.random.default_rng(5)
    x, y = rng.standard_normal(4096), rng.standard_normal(4096)
    x32, y32 = x.astype(np.float32), y.astype(np.float32)
    acc = np.float32(0)
    for a, b in zip(x32, y32):
        acc = np.float32(acc + np.float32(a * b))
    ref = float(np.dot(x32.astype(np.float64), y32.astype(np.float64)))
    ref_abs = float(np.dot(np.abs(x32).astype(np.float64), np.abs(y32).astype(np.float64)))
    e = m1([float(acc)], [ref], [ref_abs])
    assert 0 < e <= 4096 * 2.0 ** -24


def test_rel_l2_hand_values():
    # ref = [3, 4] (norm 5); got - ref = [0.3, -0.4] (norm 0.5)  ->  0.1
    assert rel_l2([3.3, 3.6], [3.0, 4.0]) == pytest.approx(0.1, rel=1e-14)
    # one large isolated deviation among many exact elements stays small: ref = ones(10000), one
    # element off by 1  ->  1 / 100
    ref = np.ones(10000)
    got = ref.copy()
    got[123] = 2.0
    assert rel_l2(got, ref) == pytest.approx(0.01, rel=1e-14)
    assert m2(got, ref) == pytest.approx(1.0, rel=1e-14)                 # where the maximum sees it whole
    assert rel_l2(np.zeros(0), np.zeros(0)) == 0.0
    assert rel_l2([0.5, 0.0], [0.0, 0.0]) == 0.5
