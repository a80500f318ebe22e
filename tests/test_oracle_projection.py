"""Pins for the oracle's N:M projection (Sec. 3.2, Eq. 3) that do not reuse its code."""
import itertools

import numpy as np
import pytest

import oracle

PATTERNS = [(1, 4), (2, 4), (3, 4), (1, 8), (2, 8), (3, 8), (4, 8), (5, 8), (7, 8)]


def brute_force_support(w, N):
    """Euclidean projection by enumeration: the support whose complement has the
    least energy; equal costs resolved towards the lexicographically smallest
    ascending index tuple."""
    M = len(w)
    best, best_cost = None, None
    for sup in itertools.combinations(range(M), N):
        cost = sum(float(w[c]) ** 2 for c in range(M) if c not in sup)
        if best is None or cost < best_cost:
            best, best_cost = sup, cost
    return best


def exact_values(rng, shape):
    # multiples of 1/8 in [-2, 2]: squares and their sums are exact in double,
    # and repeated magnitudes (ties) are frequent
    return (rng.integers(-16, 17, size=shape) / 8.0).astype(np.float32)


@pytest.mark.parametrize("N,M", PATTERNS)
def test_projection_matches_brute_force(N, M):
    rng = np.random.default_rng(100 * N + M)
    for rows, groups in [(1, 1), (2, 2), (4, 16 // M), (3, 3)]:
        for trial in range(20):
            W = exact_values(rng, (rows, groups * M))
            kept = oracle.project(W, N, M)
            for r in range(rows):
                for g in range(groups):
                    expect = brute_force_support(W[r, g * M:(g + 1) * M], N)
                    assert tuple(kept[r, g]) == expect, (W[r, g * M:(g + 1) * M], kept[r, g])


@pytest.mark.parametrize("M", [4, 8])
def test_keep_one_is_first_argmax_of_magnitude(M):
    rng = np.random.default_rng(M)
    W = exact_values(rng, (16, 8 * M))
    kept = oracle.project(W, 1, M)
    expect = np.argmax(np.abs(W).reshape(16, 8, M), axis=2)  # numpy returns the first maximum
    assert np.array_equal(kept[:, :, 0], expect)


@pytest.mark.parametrize("N,M", PATTERNS)
def test_projection_invariants(N, M):
    rng = np.random.default_rng(7)
    W = (rng.standard_normal((32, 16 * M)) * 0.02).astype(np.float32)
    W[3] = 0.0
    W[4] = 0.125
    kept = oracle.project(W, N, M).astype(int)
    assert kept.shape == (32, 16, N)
    assert np.all(kept >= 0) and np.all(kept < M)
    assert np.all(np.diff(kept, axis=2) > 0)             # ascending and distinct => exactly N positions
    A = np.abs(W).reshape(32, 16, M)
    mask = np.zeros_like(A, dtype=bool)
    np.put_along_axis(mask, kept, True, axis=2)
    assert np.all(mask.sum(axis=2) == N)
    kept_min = np.where(mask, A, np.inf).min(axis=2)
    drop_max = np.where(~mask, A, -np.inf).max(axis=2)
    assert np.all(drop_max <= kept_min)                  # nothing dropped outranks anything kept


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (4, 8)])
def test_projection_is_idempotent(N, M):
    rng = np.random.default_rng(11)
    W = exact_values(rng, (8, 8 * M))

    def apply(W):
        kept = oracle.project(W, N, M).astype(int)
        mask = np.zeros((W.shape[0], W.shape[1] // M, M), dtype=bool)
        np.put_along_axis(mask, kept, True, axis=2)
        return np.where(mask.reshape(W.shape), W, 0).astype(np.float32)

    Z = apply(W)
    assert np.array_equal(apply(Z), Z)
    # Z is feasible and no feasible point built from W's own entries is closer
    assert np.all((Z.reshape(8, -1, M) != 0).sum(axis=2) <= N)


def test_ties_zeros_and_signs():
    W = np.array([[0, 0, 0, 0, 1, 1, 1, 1, -2, 2, -2, 2, 0, -0.0, 3, -3]], np.float32)
    kept = oracle.project(W, 2, 4)[0]
    assert kept.tolist() == [[0, 1], [0, 1], [0, 1], [2, 3]]
    kept = oracle.project(W, 1, 4)[0]
    assert kept.tolist() == [[0], [0], [0], [2]]
    kept = oracle.project(W, 2, 8)[0]
    assert kept.tolist() == [[4, 5], [6, 7]]
    kept = oracle.project(W, 3, 8)[0]
    assert kept.tolist() == [[4, 5, 6], [0, 6, 7]]


def test_magnitude_not_signed_value():
    # "largest" must mean largest magnitude, or the result is not the Euclidean projection
    W = np.array([[-9.0, 1.0, 2.0, 3.0]], np.float32)
    assert oracle.project(W, 2, 4)[0].tolist() == [[0, 3]]


def test_rejects_bad_arguments_and_nonfinite():
    W = np.ones((2, 8), np.float32)
    for N, M in [(0, 4), (5, 4), (2, 5), (2, 16), (9, 8)]:
        with pytest.raises(oracle.OracleError):
            oracle.project(W, N, M)
    with pytest.raises(oracle.OracleError):
        oracle.project(np.ones((2, 6), np.float32), 2, 4)    # cols not a multiple of M
    W[1, 3] = np.nan
    with pytest.raises(oracle.OracleError):
        oracle.project(W, 2, 4)
    W[1, 3] = np.inf
    with pytest.raises(oracle.OracleError):
        oracle.compress(W, 2, 4, 8)
