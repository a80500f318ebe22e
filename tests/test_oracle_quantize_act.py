"""Pins for the oracle's activation quantiser (Sec. 5.3: 8-bit activations; Eq. 5 with offset 0 and one
scale per tensor by the largest-magnitude rule of Sec. 3.3.1).  The codes are checked against exact
rational arithmetic (the fp32 quotient rounded once, then half-to-even), the scale against numpy's
float32 division, plus the invariants a dropped clamp, a wrong rounding mode or a per-row scale would break."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2206_15014_amd import synth


def f32_quotient(x, s):
    """RN_fp32(x / s) from exact rationals: the candidates around the double quotient, the nearest one wins
    (ties to the even mantissa)."""
    exact = Fraction(float(x)) / Fraction(float(s))
    c = np.float32(float(exact))
    cands = sorted({float(np.nextafter(c, np.float32(-np.inf))), float(c), float(np.nextafter(c, np.float32(np.inf)))})
    best = min(cands, key=lambda v: (abs(Fraction(v) - exact), int(np.float32(v).view(np.uint32)) & 1))
    return Fraction(best)


def rne(fr):
    lo = fr.numerator // fr.denominator
    rem = fr - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2):
        lo += 1
    return lo


def test_codes_are_the_rounded_clamped_fp32_quotient():
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((7, 33)) * 3).astype(np.float32)
    X[2, 5] = 0.0
    X[3, :4] = [1.5, -1.5, 2.5, -2.5]
    Q, s = oracle.quantize_act(X)
    assert s == np.float32(np.abs(X).max()) / np.float32(127.0)          # one fp32 division
    for t in range(X.shape[0]):
        for k in range(X.shape[1]):
            want = max(-127, min(127, rne(f32_quotient(X[t, k], s))))
            assert int(Q[t, k]) == want, (t, k, X[t, k])


def test_half_way_quotients_round_to_even_and_the_caller_scale_is_used():
    s = np.float32(0.5)
    X = np.array([[0.25, 0.75, 1.25, -0.25, -0.75, 63.25, 63.75, 1000.0, -1000.0, 0.0]], np.float32)   # x / s = 0.5, 1.5, 2.5, ...
    Q, s_used = oracle.quantize_act(X, scale=s)
    assert s_used == s
    assert Q.tolist() == [[0, 2, 2, 0, -2, 126, 127, 127, -127, 0]]        # ties to even, then the symmetric clamp


def test_invariants():
    rng = np.random.default_rng(9)
    X = (rng.standard_normal((40, 96)) * rng.uniform(0.01, 50)).astype(np.float32)
    X[:, 7] *= 10                                                         # an outlier channel, as in the workloads
    Q, s = oracle.quantize_act(X)
    i = np.unravel_index(np.abs(X).argmax(), X.shape)
    assert abs(int(Q[i])) == 127                                          # the largest magnitude maps to the largest code
    assert np.all(np.abs(X.astype(np.float64) - float(s) * Q.astype(np.float64)) <= float(s) * 0.5 * (1 + 1e-6))
    Qn, sn = oracle.quantize_act(-X)
    assert sn == s and np.array_equal(Qn, -Q)                             # odd symmetry (half-to-even is symmetric)
    # one scale for the whole tensor, not one per row: a row of small values keeps small codes
    Y = np.vstack([np.full((1, 8), 100.0, np.float32), np.full((1, 8), 1.0, np.float32)])
    Qy, sy = oracle.quantize_act(Y)
    assert sy == np.float32(100.0) / np.float32(127.0) and Qy[1].tolist() == [1] * 8
    Qz, sz = oracle.quantize_act(np.zeros((3, 5), np.float32))
    assert sz == np.float32(1.0) and not Qz.any()


def test_agrees_with_the_numpy_generator_and_with_the_weight_quantiser():
    rng = np.random.default_rng(11)
    X = rng.standard_normal((64, 128)).astype(np.float32)
    Q, s = oracle.quantize_act(X)
    Qg, sg = synth.quantize_activations(X)                               # independent numpy implementation
    assert s == sg and np.array_equal(Q, Qg)
    for t, k in [(0, 0), (5, 17), (63, 127), (31, 64)]:
        assert int(Q[t, k]) == oracle.quantize_one(X[t, k], s, 8)


def test_errors():
    with pytest.raises(oracle.OracleError):
        oracle.quantize_act(np.array([[1.0, np.inf]], np.float32))
    with pytest.raises(oracle.OracleError):
        oracle.quantize_act(np.array([[np.nan, 1.0]], np.float32))
