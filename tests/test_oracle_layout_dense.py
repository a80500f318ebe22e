"""Pins for two parts of the oracle that the paper leaves to the implementation:

* the tiled layout of the packed bytes (a permutation of the row layout, defined in the oracle's
  source): checked against a numpy reshape / transpose of the row layout - no offset arithmetic in
  common with the C loops - and against bytes placed by hand;
* dense matrices (N = M: the "Q4" / "Q8" components of the heterogeneous configurations of
  Sec. 5.4): compress is the plain quantiser of Eq. 5 entry by entry, nothing is pruned, no index
  metadata exists, and the product equals numpy's int64 matrix product.
"""
import numpy as np
import pytest

import oracle

SCHEMES = [(2, 4, 8), (1, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (2, 8, 8), (1, 8, 8), (1, 8, 4),
           (3, 4, 8), (3, 4, 4), (4, 8, 8), (4, 8, 4), (5, 8, 4), (7, 8, 8), (4, 4, 8), (4, 4, 4), (8, 8, 8), (8, 8, 4)]


def piece_bytes(ub):
    pb = 16
    while ub % pb:
        pb //= 2
    return pb


def tiled_by_transposition(a, cols, ub):
    """[rows, cols/32 * ub] -> the tiled bytes, with numpy axis moves only."""
    rows = a.shape[0]
    r16 = -(-rows // 16) * 16
    pad = np.zeros((r16, a.shape[1]), np.uint8)
    pad[:rows] = a
    pb = piece_bytes(ub)
    # axes: row block, row in block, slice, unit in slice, piece, byte in piece
    x = pad.reshape(r16 // 16, 16, cols // 128, 4, ub // pb, pb)
    # block (row block, slice); inside: piece, unit in slice, row in block, byte
    return x.transpose(0, 2, 4, 3, 1, 5).reshape(-1)


@pytest.mark.parametrize("N,M,bits", SCHEMES)
@pytest.mark.parametrize("rows,cols", [(16, 128), (37, 256), (5, 384), (130, 768)])
def test_tiled_layout_is_the_stated_transposition(N, M, bits, rows, cols):
    rng = np.random.default_rng([N, M, bits, rows, cols])
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    vals, meta, _ = oracle.compress(W, N, M, bits)
    vt, mt = oracle.to_tiled(vals, meta, cols, N, M, bits)
    uv, um = oracle.unit_bytes(N, M, bits)
    assert np.array_equal(vt, tiled_by_transposition(vals, cols, uv))
    if um:
        assert np.array_equal(mt, tiled_by_transposition(meta, cols, um))
    else:
        assert mt.size == 0 and meta.shape == (rows, 0)
    v2, m2 = oracle.from_tiled(vt, mt, rows, cols, N, M, bits)
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)
    # the bytes are permuted, never changed: same multiset, padding rows all zero
    assert np.array_equal(np.bincount(vt, minlength=256)[1:], np.bincount(vals.ravel(), minlength=256)[1:])


def test_tiled_layout_bytes_placed_by_hand():
    # 2:4 int8, 17 rows x 256 columns: units of 16 value bytes and 4 index bytes, two slices, two
    # row blocks (the second holding one real row and fifteen rows of padding).
    rows, cols = 17, 256
    vals = np.zeros((rows, 128), np.uint8)
    meta = np.zeros((rows, 32), np.uint8)
    vals[0, 0] = 1          # row 0, unit 0, byte 0
    vals[3, 16 * 5 + 7] = 2  # row 3, unit 5 (slice 1, unit 1 of the slice), byte 7
    vals[16, 127] = 3       # row 16 (block 1, row 0), unit 7 (slice 1, unit 3), byte 15
    meta[15, 4 * 2 + 1] = 4  # row 15, unit 2, byte 1
    vt, mt = oracle.to_tiled(vals, meta, cols, 2, 4, 8)
    assert vt.size == 32 * 128 and mt.size == 32 * 32
    where = {int(i): int(vt[i]) for i in np.flatnonzero(vt)}
    assert where == {0: 1,
                     (0 * 2 + 1) * 1024 + (1 * 16 + 3) * 16 + 7: 2,
                     (1 * 2 + 1) * 1024 + (3 * 16 + 0) * 16 + 15: 3}
    assert {int(i): int(mt[i]) for i in np.flatnonzero(mt)} == {(0 * 2 + 0) * 256 + (2 * 16 + 15) * 4 + 1: 4}
    # 3:4 int8: units of 24 bytes are cut into three pieces of 8; byte 19 of a unit is byte 3 of piece 2
    v3 = np.zeros((1, 24 * 4), np.uint8)
    v3[0, 24 * 2 + 19] = 9   # row 0, unit 2
    t3, _ = oracle.to_tiled(v3, np.zeros((1, 6 * 4), np.uint8), 128, 3, 4, 8)
    assert {int(i): int(t3[i]) for i in np.flatnonzero(t3)} == {(2 * 64 + 2 * 16 + 0) * 8 + 3: 9}


def test_tiled_layout_needs_whole_slices():
    with pytest.raises(oracle.OracleError):
        oracle.to_tiled(np.zeros((4, 48), np.uint8), np.zeros((4, 12), np.uint8), 96, 2, 4, 8)


@pytest.mark.parametrize("N,M", [(4, 4), (8, 8)])
@pytest.mark.parametrize("bits", [8, 4])
def test_dense_compress_is_the_plain_quantiser(N, M, bits):
    rng = np.random.default_rng([N, bits, 3])
    rows, cols = 9, 64
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    W[4] = 0.0
    vals, meta, scales = oracle.compress(W, N, M, bits)
    assert meta.size == 0
    assert oracle.packed_sizes(rows, cols, N, M, bits) == (rows * cols * bits // 8, 0, rows * 4)
    qmax = (1 << (bits - 1)) - 1
    Wq = oracle.decompress(vals, meta, rows, cols, N, M, bits)
    for r in range(rows):
        s = oracle.row_scale(W[r], bits)
        assert scales[r] == s == (np.float32(1.0) if r == 4 else np.abs(W[r]).max() / np.float32(qmax))
        for c in range(cols):
            assert int(Wq[r, c]) == oracle.quantize_one(W[r, c], s, bits)
    # the byte format: int8 one byte per column; int4 column 2i in the low nibble of byte i
    if bits == 8:
        assert np.array_equal(vals.view(np.int8), Wq)
    else:
        lo = (vals & 15).astype(np.int16)
        hi = (vals >> 4).astype(np.int16)
        un = np.stack([lo, hi], axis=2).reshape(rows, cols)
        assert np.array_equal(np.where(un > 7, un - 16, un), Wq.astype(np.int16))
    # the dense formats of M = 4 and M = 8 are the same bytes
    other = oracle.compress(W, 12 - N, 12 - M, bits)
    assert np.array_equal(other[0], vals) and np.array_equal(other[2], scales)


@pytest.mark.parametrize("bits", [8, 4])
def test_dense_product_equals_numpy_matmul(bits):
    rng = np.random.default_rng([bits, 8])
    T, K, O = 7, 96, 11
    W = (rng.standard_normal((O, K)) * 0.02).astype(np.float32)
    X = rng.integers(-127, 128, size=(T, K)).astype(np.int8)
    vals, meta, _ = oracle.compress(W, 4, 4, bits)
    Wq = oracle.decompress(vals, meta, O, K, 4, 4, bits)
    acc = oracle.gemm_sparse(X, vals, meta, O, 4, 4, bits)
    assert np.array_equal(acc.astype(np.int64), X.astype(np.int64) @ Wq.astype(np.int64).T)
    assert np.count_nonzero(Wq) > 0.8 * Wq.size
