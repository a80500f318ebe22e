"""Pins for the oracle's requantised layer output (Eq. 4 then Eq. 5 with o = 0, 8-bit activations
of Sec. 5.3): the same chain of operations in exact rational arithmetic with every fp32 rounding
applied explicitly (a different mechanism from the C code's float arithmetic), half-way and
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


def rn32(x: Fraction) -> Fraction:
    """x rounded to the nearest fp32 number, ties to even (normal range, which is all these tests use)."""
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
    m = round_half_even(x * (1 << 23))          # 24-bit significand
    return sign * Fraction(m, 1 << 23) * (Fraction(2) ** e)


def F(v) -> Fraction:
    return Fraction(float(np.float32(v)))


def expected(acc, act_scale, scales, bias, out_scale):
    """The definition, step by step, in exact arithmetic with explicit fp32 roundings."""
    q = np.zeros(acc.shape, np.int64)
    zmax = Fraction(0)
    for o in range(acc.shape[1]):
        p = rn32(F(act_scale) * F(scales[o]))
        g = rn32(p / F(out_scale))
        h = rn32(F(bias[o]) / F(out_scale)) if bias is not None else Fraction(0)
        for t in range(acc.shape[0]):
            a = rn32(Fraction(int(acc[t, o])))              # int32 -> fp32
            z = rn32(a * g + h)                             # fused: one rounding
            zmax = max(zmax, abs(z))
            q[t, o] = min(127, max(-127, round_half_even(z)))
    return q, float(rn32(zmax * F(out_scale)))


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


def test_multiply_add_is_fused_one_rounding():
    # acc * g = 4097 * (1 + 2^-12) = 4098 + 2^-12 exactly, which fp32 cannot hold (25 bits); a
    # separately rounded product is 4098 (or 4098 + 2^-11) and the sum with -4098 then 0 (or 2^-11).
    # Fused, the sum is 2^-12 exactly.  With out_scale 2^-13 (a power of two: g and h scale exactly)
    # that is code 2; the unfused results would be 0 or 4.
    p = np.float32(1.0 + 2.0 ** -12)
    q, amax = oracle.requant(np.array([[4097]], np.int32), 1.0, np.array([p], np.float32), 2.0 ** -13,
                             np.array([-4098.0], np.float32))
    assert q.tolist() == [[2]]
    assert amax == 2.0 ** -12


def test_close_to_the_weight_quantiser_on_the_dequantised_value():
    # Eq. 5 is one function: the codes must be those the (separately pinned) weight quantiser gives
    # for the dequantised value and the same scale at 8 bits, up to the one-step difference that
    # folding the division into the column constants can make next to a half-way point.
    rng = np.random.default_rng(11)
    acc = rng.integers(-3_000_000, 3_000_000, size=(4, 33)).astype(np.int32)
    scales = (rng.random(33) * 1e-4 + 2e-5).astype(np.float32)
    bias = (rng.standard_normal(33) * 0.2).astype(np.float32)
    sx, so = np.float32(0.0123), np.float32(0.0371)
    q, amax = oracle.requant(acc, sx, scales, so, bias)
    f32, _ = oracle.dequant(acc, sx, scales, bias)
    differ = 0
    for t in range(4):
        for o in range(33):
            want = oracle.quantize_one(float(f32[t, o]), float(so), 8)
            assert abs(int(q[t, o]) - want) <= 1
            differ += int(q[t, o]) != want
    assert differ <= 2
    assert np.count_nonzero(np.abs(q.astype(int)) < 127) > 60      # most codes inside the range: the comparison means something
    assert abs(amax - np.abs(f32).max()) <= np.abs(f32).max() * 2.0 ** -21


def test_rejects_bad_scale():
    acc = np.zeros((1, 1), np.int32)
    for s in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(oracle.OracleError):
            oracle.requant(acc, 1.0, np.ones(1, np.float32), s)
