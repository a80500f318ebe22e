"""Pins for the oracle's ADMM Z-update Z = Pi(W + U) (Sec. 3.1, Eq. 3 on W + U; quantisation
constraint after the sparsity one with the ADMM-Max scale of Sec. 3.3.1; scale groups of output
neurons, Sec. 4) and the dual update U + W - Z."""
import itertools

import numpy as np
import pytest

import oracle

PATTERNS = [(2, 4), (1, 4), (3, 4), (2, 8), (4, 8), (1, 8)]


def brute_force_projection(V, N, M):
    """Euclidean projection onto 'at most N non-zeros per group of M' by trying every support:
    the closest point keeps V on the support that carries the most squared magnitude."""
    Z = np.zeros_like(V)
    for r in range(V.shape[0]):
        for g in range(V.shape[1] // M):
            grp = V[r, g * M:(g + 1) * M].astype(np.float64)
            best, best_err = None, None
            for sup in itertools.combinations(range(M), N):          # ascending: ties go to the lower columns
                z = np.zeros(M)
                z[list(sup)] = grp[list(sup)]
                err = float(np.sum((grp - z) ** 2))
                if best_err is None or err < best_err:
                    best, best_err = z, err
            Z[r, g * M:(g + 1) * M] = best
    return Z


@pytest.mark.parametrize("N,M", PATTERNS)
def test_sparsity_only_is_the_euclidean_projection_of_w_plus_u(N, M):
    rng = np.random.default_rng(31 * N + M)
    rows, cols = 5, 6 * M
    W = (rng.integers(-40, 41, size=(rows, cols)) / 8.0).astype(np.float32)      # eighths: sums and squares exact
    U = (rng.integers(-40, 41, size=(rows, cols)) / 8.0).astype(np.float32)
    Z, Uo, scales = oracle.admm_project(W, U, N, M, 0, 1)
    assert scales is None
    V = W + U
    ref = brute_force_projection(V, N, M)
    # equal squared distance is what the projection fixes; which of several equally good supports is
    # the tie rule's business, pinned separately
    assert np.allclose(np.sum((V - Z) ** 2, axis=1), np.sum((V - ref) ** 2, axis=1), rtol=0, atol=0)
    assert np.all((Z == 0) | (Z == V))
    assert np.all(np.count_nonzero(Z.reshape(rows, -1, M), axis=2) <= N)
    assert np.array_equal(Uo, V - Z)                        # the dual update
    Z0, Uo0, _ = oracle.admm_project(V, None, N, M, 0, 1)    # U absent = U zero
    assert np.array_equal(Z0, Z) and np.array_equal(Uo0, Uo)
    Z2, Uo2, _ = oracle.admm_project(Z, None, N, M, 0, 1)    # a point of the set projects onto itself
    assert np.array_equal(Z2, Z) and not Uo2.any()


def test_tie_rule_and_signed_zeros():
    W = np.array([[1, -1, 1, -1, 0, 0, 0, 0, 2, 2, -3, 3]], np.float32)
    Z, Uo, _ = oracle.admm_project(W, None, 2, 4, 0, 1)
    assert Z.tolist() == [[1, -1, 0, 0, 0, 0, 0, 0, 0, 0, -3, 3]]
    assert Uo.tolist() == [[0, 0, 1, -1, 0, 0, 0, 0, 2, 2, 0, 0]]
    assert not np.signbit(Z[0, 2:10]).any()                 # pruned positions are +0


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 8), (2, 8, 4), (4, 8, 8)])
def test_with_row_scales_it_is_compress_then_dequantise(N, M, bits):
    """rows_per_scale = 1 must give s[o] * (decompressed codes of nm_compress): two separately
    pinned paths of the oracle (byte format decoder, quantiser) meet here."""
    rng = np.random.default_rng(100 + 7 * N + M + bits)
    rows, cols = 9, 10 * M
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    U = (rng.standard_normal((rows, cols)) * 0.004).astype(np.float32)
    V = (W + U).astype(np.float32)
    Z, Uo, scales = oracle.admm_project(W, U, N, M, bits, 1)
    vals, meta, s_ref = oracle.compress(V, N, M, bits)
    codes = oracle.decompress(vals, meta, rows, cols, N, M, bits).astype(np.float32)
    assert np.array_equal(scales, s_ref)
    assert np.array_equal(Z, (s_ref[:, None] * codes).astype(np.float32))
    assert np.array_equal(Uo, (V - Z).astype(np.float32))
    kept = oracle.project(V, N, M)                          # the support is that of Eq. 3 on V
    mask = np.zeros((rows, cols), bool)
    for r in range(rows):
        for g in range(cols // M):
            mask[r, g * M + kept[r, g]] = True
    assert not Z[~mask].any()
    assert np.all(np.abs(V[mask] - Z[mask]) <= np.repeat(scales, cols * N // M) / 2 * (1 + 1e-6))


@pytest.mark.parametrize("rps", [2, 32, 70, 1000])
def test_scale_groups_of_rows(rps):
    rng = np.random.default_rng(rps)
    rows, cols, N, M, bits = 70, 24, 2, 4, 8                # 70 rows: the last group of 32 is 6 rows long
    W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
    Z, Uo, scales = oracle.admm_project(W, None, N, M, bits, rps)
    want = np.zeros(rows, np.float32)
    for r0 in range(0, rows, rps):
        want[r0:r0 + rps] = np.float32(np.abs(W[r0:r0 + rps]).max()) / np.float32(127.0)
    assert np.array_equal(scales, want)                     # ADMM-Max, one scale per group of rows
    codes = Z / scales[:, None]
    assert np.all(np.abs(codes - np.rint(codes)) < 1e-4) and np.abs(np.rint(codes)).max() == 127
    for r0 in range(0, rows, rps):                          # the group's largest entry survives at the largest code
        blk = np.abs(np.rint(codes[r0:r0 + rps]))
        assert blk.max() == 127
    nz = Z != 0
    assert np.all(np.abs(W[nz] - Z[nz]) <= (scales[:, None] * np.ones_like(W))[nz] / 2 * (1 + 1e-6))
    assert np.array_equal(Uo, (W - Z).astype(np.float32))
    # a whole-matrix group is the same as one huge rows_per_scale
    if rps == 1000:
        Zb, _, sb = oracle.admm_project(W, None, N, M, bits, rows)
        assert np.array_equal(Zb, Z) and np.array_equal(sb, scales)


def test_zero_group_and_errors():
    W = np.zeros((4, 8), np.float32)
    W[2:, :] = np.array([1, 2, 3, 4, -4, -3, -2, -1], np.float32)
    Z, Uo, scales = oracle.admm_project(W, None, 2, 4, 8, 2)
    assert scales.tolist() == [1.0, 1.0, np.float32(4.0) / np.float32(127.0), np.float32(4.0) / np.float32(127.0)]
    assert not Z[:2].any() and not Uo[:2].any()
    with pytest.raises(oracle.OracleError):
        oracle.admm_project(W, None, 2, 4, 8, 0)
    with pytest.raises(oracle.OracleError):
        oracle.admm_project(W, None, 5, 4, 8, 1)
    bad = W.copy()
    bad[0, 0] = np.inf
    with pytest.raises(oracle.OracleError):
        oracle.admm_project(bad, None, 2, 4, 8, 1)


@pytest.mark.parametrize("N,M,bits,rps", [(2, 4, 8, 32), (2, 4, 4, 5), (1, 4, 8, 70), (2, 8, 4, 32), (4, 8, 8, 2)])
def test_grouped_compress_is_the_packed_form_of_the_projection(N, M, bits, rps):
    """One scale per group of rows in the packed format: scales from numpy group maxima, codes
    that dequantise to exactly the Z of the ADMM projection (bit for bit), and, entry by entry,
    the quantiser applied with the group's scale at the positions Eq. 3 keeps."""
    rng = np.random.default_rng([N, M, bits, rps])
    rows, cols = 70, 12 * M
    W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
    W[3 * (rps > 1):3 * (rps > 1) + min(rps, 4)] = 0.0       # zero rows; a whole zero group when the group is small
    vals, meta, scales = oracle.compress_grouped(W, N, M, bits, rps)
    qmax = np.float32((1 << (bits - 1)) - 1)
    want = np.zeros(rows, np.float32)
    for r0 in range(0, rows, rps):
        m = np.float32(np.abs(W[r0:r0 + rps]).max())
        want[r0:r0 + rps] = np.float32(1.0) if m == 0 else m / qmax
    assert np.array_equal(scales, want)
    codes = oracle.decompress(vals, meta, rows, cols, N, M, bits)
    Z, _, s2 = oracle.admm_project(W, None, N, M, bits, rps)
    assert np.array_equal(s2, scales)
    assert np.array_equal((scales[:, None] * codes.astype(np.float32)).astype(np.float32).view(np.uint32), Z.view(np.uint32))
    kept = oracle.project(W, N, M)
    for r in range(0, rows, 7):
        for g in range(cols // M):
            for j in range(N):
                c = g * M + int(kept[r, g, j])
                assert codes[r, c] == oracle.quantize_one(W[r, c], scales[r], bits)
    # rows_per_scale = 1 is the library's default granularity
    v1, m1, s1 = oracle.compress_grouped(W, N, M, bits, 1)
    v0, m0, s0 = oracle.compress(W, N, M, bits)
    assert np.array_equal(v1, v0) and np.array_equal(m1, m0) and np.array_equal(s1, s0)
