"""The quotient route of the compress kernels, checked on the CPU: for one divisor s and many
dividends w, q0 = RN(w*y) with y = RN(1/s), followed by two fused-multiply-add corrections
q <- RN(q + RN(w - s*q)*y), gives the correctly rounded fp32 quotient RN(w/s) (Markstein's
theorem on division by fused multiply-add, applied after the first correction has brought q
within an ulp).  The fused operations are emulated exactly (double products of fp32 numbers are
exact; sums go through an error-free transformation and, on exact ties of the double sum, through
rational arithmetic) and compared with the division operator on dividends placed on and within a
few ulps of the half-way points (k + 1/2)*s, where the integer code hinges on the last bit of the
quotient, for divisors whose significands include all ones and all zeros."""
from fractions import Fraction

import numpy as np

f32, f64 = np.float32, np.float64


def rn32_of_sum(a64, b64):
    """RN32(a + b), a and b float64 arrays whose exact sum need not be a float64."""
    hi = a64 + b64
    bb = hi - a64
    err = (a64 - (hi - bb)) + (b64 - bb)            # a + b = hi + err exactly (TwoSum)
    r = hi.astype(f32)
    d = hi - r.astype(f64)
    half_ulp = np.spacing(np.abs(r)).astype(f64) / 2
    below = np.spacing(np.nextafter(np.abs(r), f32(0))).astype(f64) / 2      # the spacing shrinks below a power of two
    tie = (np.abs(d) == half_ulp) | (np.abs(d) == below)
    for i in np.nonzero(tie & (err != 0))[0]:        # the double sum sits on a tie that the exact sum does not
        exact = Fraction(float(a64[i])) + Fraction(float(b64[i]))
        cands = [np.nextafter(r[i], f32(-np.inf)), r[i], np.nextafter(r[i], f32(np.inf))]
        r[i] = min(cands, key=lambda c: (abs(Fraction(float(c)) - exact), int(f32(c).view(np.uint32)) & 1))
    return r


def fma32(a, b, c):
    return rn32_of_sum(a.astype(f64) * b.astype(f64), c.astype(f64))


def quotient_by_reciprocal(w, s):
    y = (f32(1) / s).astype(f32)
    q0 = (w * y).astype(f32)
    q1 = fma32(fma32(-s, q0, w), y, q0)
    return fma32(fma32(-s, q1, w), y, q1)


def divisors(rng, n):
    mant = rng.integers(0, 1 << 23, n, dtype=np.uint32)
    mant[: n // 50] = (1 << 23) - 1 - rng.integers(0, 4, n // 50)          # significands of all ones, and next to it
    mant[n // 50: n // 25] = rng.integers(0, 4, n // 50)                     # of all zeros, and next to it
    expo = rng.integers(127 - 60, 127 + 61, n, dtype=np.uint32)              # the range in which the kernel takes this route
    return ((expo << 23) | mant).view(f32)


def test_dividends_around_half_way_points():
    rng = np.random.default_rng(1)
    n = 1_000_000
    s = divisors(rng, n)
    k = rng.integers(-127, 127, n).astype(f64) + 0.5
    w = (k * s.astype(f64)).astype(f32)
    w = (w.view(np.int32) + rng.integers(-3, 4, n).astype(np.int32)).view(f32)
    assert np.array_equal(quotient_by_reciprocal(w, s).view(np.uint32), (w / s).astype(f32).view(np.uint32))


def test_random_dividends_in_the_code_range():
    rng = np.random.default_rng(2)
    n = 1_000_000
    s = divisors(rng, n)
    w = (rng.uniform(-127.2, 127.2, n) * s.astype(f64)).astype(f32)
    assert np.array_equal(quotient_by_reciprocal(w, s).view(np.uint32), (w / s).astype(f32).view(np.uint32))
