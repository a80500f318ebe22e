"""Pins for the oracle's second scale rule (Sec. 3.3.1, "ADMM-Dist": the scale minimising the L2
distance between quantised and raw parameters).  The paper states the criterion only; what the
oracle adds (a candidate grid from the max-rule scale down to half of it, the error taken over the
kept entries) is this build's reading, so these pins hold the implementation to that reading and
to what the criterion itself fixes: a closed-form case with a sharp threshold between two
candidates, the least error among all candidates by an independent numpy evaluation, never worse
than the max rule, additivity of the error over the rows of a group, and the degenerate cases."""
import numpy as np
import pytest

import oracle


def numpy_errors(W, N, M, bits, smax, C):
    """Error of every candidate, numpy float64, with the kept mask from the (separately pinned) projection."""
    kept = oracle.project(W, N, M)
    rows, cols = W.shape
    mask = np.zeros((rows, cols // M, M), bool)
    np.put_along_axis(mask, kept.astype(np.int64), True, axis=2)
    w = W.reshape(rows, cols // M, M)[mask].astype(np.float32)
    qmax = (1 << (bits - 1)) - 1
    out = []
    for c in range(C // 2, C + 1):
        s = np.float32(np.float32(smax * np.float32(c)) / np.float32(C))
        q = np.clip(np.rint(w / s), -qmax, qmax)
        out.append(float(np.sum((w.astype(np.float64) - np.float64(s) * q.astype(np.float64)) ** 2)))
    return np.array(out)


def test_closed_form_threshold_between_two_candidates():
    # Dense 8-bit row: one entry of 127 (max-rule scale exactly 1) and n half-integers below 64.
    # Scale 1 rounds every half-integer to the even neighbour: error n / 4.  Scale 1/2 holds them
    # exactly but clips 127 to 63.5: error 63.5^2 = 4032.25.  With two candidates (1/2 and 1) the
    # half scale wins exactly when n / 4 > 4032.25, i.e. from n = 16130 on.
    for n, want in [(16123, 1.0), (16127, 1.0), (16131, 0.5), (16135, 0.5)]:
        row = np.empty(n + 1, np.float32)
        row[0] = 127.0
        row[1:] = (np.arange(n) % 63) + 0.5
        assert (n + 1) % 4 == 0
        s, err = oracle.dist_scales(row[None, :], 4, 4, 8, 1, 2)
        assert s[0] == np.float32(want), n
        assert err[0].tolist() == [4032.25, n / 4.0]


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (4, 4, 4), (3, 4, 8)])
def test_least_error_among_the_candidates(N, M, bits):
    rng = np.random.default_rng([N, M, bits, 6])
    rows, cols, C = 12, 256, 32
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    W[3] *= np.linspace(0.1, 3.0, cols).astype(np.float32)      # a row with a heavy tail: a smaller scale pays
    W[5] = 0.0
    qmax = (1 << (bits - 1)) - 1
    for rps in (1, 4, 5, 100):
        s, err = oracle.dist_scales(W, N, M, bits, rps, C)
        for gi, r0 in enumerate(range(0, rows, rps)):
            blk = W[r0:r0 + rps]
            amax = np.abs(blk).max()
            smax = np.float32(1.0) if amax == 0 else np.float32(amax) / np.float32(qmax)
            ref = numpy_errors(blk, N, M, bits, smax, C)
            assert np.allclose(err[gi], ref, rtol=1e-12, atol=0)
            best = C // 2 + int(np.max(np.flatnonzero(err[gi] == err[gi].min())))     # ties: the larger scale
            want = np.float32(np.float32(smax * np.float32(best)) / np.float32(C))
            assert np.all(s[r0:r0 + rps] == want)
            assert err[gi].min() <= err[gi][-1]                  # never worse than the max rule (c = C)
    s1, e1 = oracle.dist_scales(W, N, M, bits, 1, C)
    assert s1[5] == 1.0 and not e1[5].any()                      # an all-zero row: scale 1, as under the max rule
    if bits == 4:
        assert np.any(s1 < np.abs(W).max(axis=1) / np.float32(qmax))   # at 4 bits a scale below the max rule does win somewhere
    # the error of a group is the sum of its rows' errors at the same candidate scale
    s4, e4 = oracle.dist_scales(W[:4] * 0 + W[0], N, M, bits, 4, C)     # four identical rows: same s_max
    _, e0 = oracle.dist_scales(W[:1], N, M, bits, 1, C)
    assert np.allclose(e4[0], 4 * e0[0], rtol=1e-13)


def test_compress_with_given_scales_is_the_quantiser_at_the_kept_positions():
    rng = np.random.default_rng(8)
    W = (rng.standard_normal((9, 64)) * 0.02).astype(np.float32)
    s, _ = oracle.dist_scales(W, 2, 4, 4, 3, 16)
    vals, meta = oracle.compress_scaled(W, 2, 4, 4, s)
    Wq = oracle.decompress(vals, meta, 9, 64, 2, 4, 4)
    kept = oracle.project(W, 2, 4)
    for r in range(9):
        for g in range(16):
            for j in range(2):
                c = g * 4 + int(kept[r, g, j])
                assert int(Wq[r, c]) == oracle.quantize_one(W[r, c], s[r], 4)
    assert np.count_nonzero(Wq) <= 9 * 32
    # with the max-rule scales it is compress itself
    v0, m0, s0 = oracle.compress(W, 2, 4, 4)
    v1, m1 = oracle.compress_scaled(W, 2, 4, 4, s0)
    assert np.array_equal(v0, v1) and np.array_equal(m0, m1)


def test_errors():
    W = np.zeros((4, 8), np.float32)
    for bad in (0, 1, 3, 66):
        with pytest.raises(oracle.OracleError):
            oracle.dist_scales(W, 2, 4, 8, 1, bad)
    with pytest.raises(oracle.OracleError):
        oracle.dist_scales(W, 2, 4, 8, 0, 8)
    W[0, 0] = np.nan
    with pytest.raises(oracle.OracleError):
        oracle.dist_scales(W, 2, 4, 8, 1, 8)
