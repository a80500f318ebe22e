"""Pins for the oracle's requantised layer output (Eq. 4 then Eq. 5 with o = 0, 8-bit activations
of Sec. 5.3): exact rational arithmetic on inputs whose fp32 steps are exact, half-way and
saturation cases, the int32 -> fp32 conversion, and the single rounding of the fused multiply-add."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def round_half_even(x: Fraction) -> int:
    f = x.numerator // x.denominator            # floor
    r = x - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        return f + 1
    return f


def expected(acc, act_scale, scales, bias, out_scale):
    """Exact rationals: valid whenever every fp32 step of the definition is exact."""
    q = np.zeros(acc.shape, np.int64)
    amax = Fraction(0)
    for t in range(acc.shape[0]):
        for o in range(acc.shape[1]):
            y = Fraction(int(acc[t, o])) * Fraction(float(act_scale)) * Fraction(float(scales[o]))
            if bias is not None:
                y += Fraction(float(bias[o]))
            amax = max(amax, abs(y))
            q[t, o] = min(127, max(-127, round_half_even(y / Fraction(float(out_scale)))))
    return q, float(amax)


def test_exact_cases_against_rational_arithmetic():
    rng = np.random.default_rng(5)
    T, O = 9, 14                                           # different: a transposed index shows
    acc = rng.integers(-(1 << 18), 1 << 18, size=(T, O)).astype(np.int32)
    scales = (2.0 ** rng.integers(-9, -5, size=O)).astype(np.float32)       # powers of two: products exact
    bias = (rng.integers(-64, 64, size=O) * 2.0 ** -4).astype(np.float32)   # on the grid of the products
    for act_scale, out_scale in [(0.25, 2.0), (0.5, 0.75), (1.0, 3.0)]:
        # 0.75 and 3.0 are not powers of two, but quotients that land on n + 1/2 exactly are still
        # representable (few significant bits), and everything else rounds the same way in fp32 and
        # exactly unless it lies within half an fp32 ulp of a half-way point, which these grids exclude.
        q, amax = oracle.requant(acc, act_scale, scales, out_scale, bias)
        eq, eamax = expected(acc, act_scale, scales, bias, out_scale)
        assert np.array_equal(q.astype(np.int64), eq)
        assert amax == eamax
        q0, amax0 = oracle.requant(acc, act_scale, scales, out_scale, None)
        eq0, eamax0 = expected(acc, act_scale, scales, None, out_scale)
        assert np.array_equal(q0.astype(np.int64), eq0) and amax0 == eamax0
    assert q.dtype == np.int8 and q.shape == (T, O)


def test_half_way_cases_round_to_even_and_codes_saturate_at_127():
    acc = np.array([[1, 3, 5, 7, -1, -3, -5, 253, 255, 257, -255, -257, 100000, -100000]], np.int32)
    scales = np.ones(acc.shape[1], np.float32)
    q, amax = oracle.requant(acc, 0.5, scales, 1.0)        # y = acc / 2: .5, 1.5, 2.5, ...
    assert q.tolist() == [[0, 2, 2, 4, 0, -2, -2, 126, 127, 127, -127, -127, 127, -127]]
    assert amax == 50000.0
    # the scale divides: the same y with out_scale 2 halves the codes (ties again to even)
    q2, _ = oracle.requant(np.array([[2, 6, 10, -6]], np.int32), 0.5, np.ones(4, np.float32), 2.0)
    assert q2.tolist() == [[0, 2, 2, -2]]                  # 0.5, 1.5, 2.5, -1.5


def test_bias_enters_before_the_quantiser_and_per_column():
    acc = np.array([[10, 10, 10], [-10, -10, -10]], np.int32)
    scales = np.array([1.0, 2.0, 0.5], np.float32)
    bias = np.array([0.0, -20.0, 100.0], np.float32)
    q, amax = oracle.requant(acc, 1.0, scales, 1.0, bias)
    assert q.tolist() == [[10, 0, 105], [-10, -40, 95]]
    assert amax == 105.0


def test_int32_to_fp32_conversion_rounds_to_nearest_even():
    # 2^24 + 1 is not an fp32 number: it becomes 2^24 (tie, even), 2^24 + 3 becomes 2^24 + 4
    acc = np.array([[(1 << 24) + 1, (1 << 24) + 3, -((1 << 24) + 3)]], np.int32)
    q, amax = oracle.requant(acc, 1.0, np.ones(3, np.float32), float(1 << 18))
    # y / out_scale = 64 exactly for the first, 64 + 4/2^18 for the second: both round to 64
    assert q.tolist() == [[64, 64, -64]]
    assert amax == float((1 << 24) + 4)


def test_multiply_add_is_fused_one_rounding():
    # acc * p = 4097 * (1 + 2^-12) = 4098 + 2^-12 exactly, which fp32 cannot hold (25 bits); a
    # separately rounded product is 4098 (or 4098 + 2^-11) and the sum with -4098 then 0 (or 2^-11).
    # Fused, the sum is 2^-12 exactly, i.e. code 2 at out_scale 2^-13 (the others: 0 or 4).
    p = np.float32(1.0 + 2.0 ** -12)
    q, amax = oracle.requant(np.array([[4097]], np.int32), 1.0, np.array([p], np.float32), 2.0 ** -13,
                             np.array([-4098.0], np.float32))
    assert q.tolist() == [[2]]
    assert amax == 2.0 ** -12


def test_agrees_with_the_weight_quantiser_on_the_dequantised_value():
    # Eq. 5 is one function: the output quantiser applied to y must give what the (separately
    # pinned) weight quantiser gives for the same value and scale at 8 bits.
    rng = np.random.default_rng(11)
    acc = rng.integers(-3_000_000, 3_000_000, size=(4, 33)).astype(np.int32)
    scales = (rng.random(33) * 1e-3 + 1e-4).astype(np.float32)
    bias = (rng.standard_normal(33) * 0.02).astype(np.float32)
    sx, so = np.float32(0.0123), np.float32(0.0371)
    q, amax = oracle.requant(acc, sx, scales, so, bias)
    f32, _ = oracle.dequant(acc, sx, scales, bias)
    # the double-rounded fp32 of nmo_dequant and the fused fp32 value differ by at most one ulp
    mism = 0
    for t in range(4):
        for o in range(33):
            want = oracle.quantize_one(float(f32[t, o]), float(so), 8)
            mism += int(abs(int(q[t, o]) - want) > 1)
            if abs(f32[t, o]) / so < 126.0:
                assert abs(int(q[t, o]) - want) <= 1
    assert mism == 0
    assert abs(amax - np.abs(f32).max()) <= np.abs(f32).max() * 2.0 ** -22


def test_rejects_bad_scale():
    acc = np.zeros((1, 1), np.int32)
    for s in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(oracle.OracleError):
            oracle.requant(acc, 1.0, np.ones(1, np.float32), s)
