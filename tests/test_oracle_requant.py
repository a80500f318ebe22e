"""Pins for the oracle's requantised layer output (Eq. 4 then Eq. 5 with o = 0, 8-bit activations
of Sec. 5.3): the definition in exact rational arithmetic (the value of Eq. 4 rounded once to
fp32, the quotient of Eq. 5 rounded once to fp32, then to the nearest integer, ties to even - a
different mechanism from the C code's floating-point operations), half-way and saturation cases,
the single rounding of the dequantised value, and agreement with the separately pinned weight
quantiser and dequantiser."""
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


def rn(x: Fraction, sig: int) -> Fraction:
    """x rounded to the nearest binary floating-point number with a `sig`-bit significand, ties to
    even (normal range, which is all these tests use)."""
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    x = abs(x)
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    assert -126 <= e <= 127
    m = round_half_even(x * (1 << (sig - 1)))
    return sign * Fraction(m, 1 << (sig - 1)) * (Fraction(2) ** e)


def rn32(x: Fraction) -> Fraction:
    return rn(x, 24)


def F(v) -> Fraction:
    return Fraction(float(np.float32(v)))


def expected(acc, act_scale, scales, bias, out_scale):
    """Eq. 4, then Eq. 5, in exact arithmetic.  The dequantised value is rounded to fp32 once;
    on the way the oracle holds it in double, whose own roundings (53 bits) are applied too, so
    that a value next to an fp32 rounding boundary is decided as the C code decides it."""
    q = np.zeros(acc.shape, np.int64)
    ymax = Fraction(0)
    for t in range(acc.shape[0]):
        for o in range(acc.shape[1]):
            y = rn(rn(Fraction(int(acc[t, o])) * F(act_scale), 53) * F(scales[o]), 53)
            if bias is not None:
                y = rn(y + F(bias[o]), 53)
            y = rn32(y)
            ymax = max(ymax, abs(y))
            q[t, o] = min(127, max(-127, round_half_even(rn32(y / F(out_scale)))))
    return q, float(ymax)


def test_random_cases_against_exact_arithmetic_with_explicit_roundings():
    rng = np.random.default_rng(5)
    T, O = 9, 14                                           # different: a transposed index shows
    acc = rng.integers(-3_000_000, 3_000_000, size=(T, O)).astype(np.int32)
    acc[0, 0], acc[1, 1] = (1 << 25) + 3, -((1 << 24) + 1)  # not fp32 numbers
    scales = (rng.random(O) * 1e-4 + 2e-5).astype(np.float32)      # codes spread over the whole range, some saturate
    bias = (rng.standard_normal(O) * 0.5).astype(np.float32)
    for act_scale, out_scale in [(0.0123, 0.0371), (0.35, 1.3), (1.0, 3.0)]:
        q, amax = oracle.requant(acc, act_scale, scales, out_scale, bias)
        eq, eamax = expected(acc, act_scale, scales, bias, out_scale)
        assert np.array_equal(q.astype(np.int64), eq)
        assert amax == eamax
        q0, amax0 = oracle.requant(acc, act_scale, scales, out_scale, None)
        eq0, eamax0 = expected(acc, act_scale, scales, None, out_scale)
        assert np.array_equal(q0.astype(np.int64), eq0) and amax0 == eamax0
        assert np.any(q != q0)                             # the bias matters in these cases
        assert 20 < np.count_nonzero(np.abs(q0.astype(int)) < 127) and np.any(np.abs(q0.astype(int)) == 127)
    assert q.dtype == np.int8 and q.shape == (T, O)


def test_half_way_cases_round_to_even_and_codes_saturate_at_127():
    acc = np.array([[1, 3, 5, 7, -1, -3, -5, 253, 255, 257, -255, -257, 100000, -100000]], np.int32)
    scales = np.ones(acc.shape[1], np.float32)
    q, amax = oracle.requant(acc, 0.5, scales, 1.0)        # z = acc / 2: .5, 1.5, 2.5, ...
    assert q.tolist() == [[0, 2, 2, 4, 0, -2, -2, 126, 127, 127, -127, -127, 127, -127]]
    assert amax == 50000.0
    # the scale divides: the same values with out_scale 2 halve (ties again to even)
    q2, amax2 = oracle.requant(np.array([[2, 6, 10, -6]], np.int32), 0.5, np.ones(4, np.float32), 2.0)
    assert q2.tolist() == [[0, 2, 2, -2]]                  # 0.5, 1.5, 2.5, -1.5
    assert amax2 == 5.0                                    # max |y| is reported in the units of y


def test_bias_enters_before_the_rounding_and_per_column():
    acc = np.array([[10, 10, 10], [-10, -10, -10]], np.int32)
    scales = np.array([1.0, 2.0, 0.5], np.float32)
    bias = np.array([0.0, -20.0, 100.0], np.float32)
    q, amax = oracle.requant(acc, 1.0, scales, 1.0, bias)
    assert q.tolist() == [[10, 0, 105], [-10, -40, 95]]
    assert amax == 105.0
    q, _ = oracle.requant(acc, 1.0, scales, 0.5, bias)     # half the scale, twice the codes
    assert q.tolist() == [[20, 0, 127], [-20, -80, 127]]


def test_int32_to_fp32_conversion_rounds_to_nearest_even():
    # 2^24 + 1 is not an fp32 number: it becomes 2^24 (tie, even), 2^24 + 3 becomes 2^24 + 4
    acc = np.array([[(1 << 24) + 1, (1 << 24) + 3, -((1 << 24) + 3)]], np.int32)
    q, amax = oracle.requant(acc, 1.0, np.ones(3, np.float32), float(1 << 18))
    assert q.tolist() == [[64, 64, -64]]
    assert amax == float((1 << 24) + 4)


def test_product_and_bias_are_summed_before_the_single_rounding():
    # acc * s = 4097 * (1 + 2^-12) = 4098 + 2^-12 exactly, which fp32 cannot hold (25 bits); a
    # product rounded to fp32 on its own is 4098 (or 4098 + 2^-11) and the sum with -4098 then 0
    # (or 2^-11).  Formed in double and rounded once, the sum is 2^-12 exactly.  With out_scale
    # 2^-13 that is code 2; the separately rounded results would be 0 or 4.
    p = np.float32(1.0 + 2.0 ** -12)
    q, amax = oracle.requant(np.array([[4097]], np.int32), 1.0, np.array([p], np.float32), 2.0 ** -13,
                             np.array([-4098.0], np.float32))
    assert q.tolist() == [[2]]
    assert amax == 2.0 ** -12


def test_is_the_weight_quantiser_applied_to_the_dequantised_value():
    # Eq. 5 is one function: the codes are those the (separately pinned) weight quantiser gives for
    # the (separately pinned) dequantised value and the same scale at 8 bits, entry by entry, and
    # the statistic is the largest magnitude of that dequantised value.
    rng = np.random.default_rng(11)
    acc = rng.integers(-3_000_000, 3_000_000, size=(4, 33)).astype(np.int32)
    scales = (rng.random(33) * 1e-4 + 2e-5).astype(np.float32)
    bias = (rng.standard_normal(33) * 0.2).astype(np.float32)
    sx, so = np.float32(0.0123), np.float32(0.0371)
    q, amax = oracle.requant(acc, sx, scales, so, bias)
    f32, _ = oracle.dequant(acc, sx, scales, bias)
    for t in range(4):
        for o in range(33):
            assert int(q[t, o]) == oracle.quantize_one(float(f32[t, o]), float(so), 8)
    assert np.count_nonzero(np.abs(q.astype(int)) < 127) > 60      # most codes inside the range: the comparison means something
    assert amax == float(np.abs(f32).max())


def test_rejects_bad_scale():
    acc = np.zeros((1, 1), np.int32)
    for s in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(oracle.OracleError):
            oracle.requant(acc, 1.0, np.ones(1, np.float32), s)
