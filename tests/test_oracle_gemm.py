"""Pins for the oracle's sparse integer product (Sec. 5.3) and dequantisation (Eq. 4)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2206_15014_amd import synth

SCHEMES = [(2, 4, 8), (1, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (3, 4, 8), (4, 8, 4)]


@pytest.mark.parametrize("N,M,bits", SCHEMES)
def test_sparse_product_equals_dense_product_and_numpy(N, M, bits):
    rng = np.random.default_rng(17 * N + M + bits)
    T, K, O = 13, 12 * M, 21                                    # all different: a swapped operand shows
    W = (rng.standard_normal((O, K)) * 0.02).astype(np.float32)
    X = rng.integers(-127, 128, size=(T, K)).astype(np.int8)
    vals, meta, _ = oracle.compress(W, N, M, bits)
    Wq = oracle.decompress(vals, meta, O, K, N, M, bits)
    acc = oracle.gemm_sparse(X, vals, meta, O, N, M, bits)
    assert acc.shape == (T, O)
    assert np.array_equal(acc, oracle.gemm_dense(X, Wq))
    assert np.array_equal(acc.astype(np.int64), X.astype(np.int64) @ Wq.astype(np.int64).T)


def test_hand_cases():
    # K = M, one token, one neuron: kept columns 1 and 3 with codes -127 and 64
    W = np.array([[1, -127, 3, 64]], np.float32)
    vals, meta, _ = oracle.compress(W, 2, 4, 8)
    X = np.array([[10, 2, -50, -3]], np.int8)
    assert oracle.gemm_sparse(X, vals, meta, 1, 2, 4, 8).tolist() == [[2 * -127 + -3 * 64]]
    # extreme codes at the longest reduction of the workloads stay inside int32
    K = 4096
    W = np.ones((1, K), np.float32)
    vals, meta, _ = oracle.compress(W, 2, 4, 8)
    X = np.full((1, K), -127, np.int8)
    assert oracle.gemm_sparse(X, vals, meta, 1, 2, 4, 8)[0, 0] == -127 * 127 * (K // 2)


def test_dequant_special_cases():
    acc = np.array([[3, -5, 0, 2 ** 24 + 1]], np.int32)
    ones = np.ones(4, np.float32)
    f32, b16 = oracle.dequant(acc, 1.0, ones)
    assert np.array_equal(f32, acc.astype(np.float32))          # identity scales: y == float(acc)
    f32, _ = oracle.dequant(acc[:, :2], 0.5, np.array([0.25, 2.0], np.float32),
                            np.array([1.0, -1.0], np.float32))
    assert f32.tolist() == [[1.375, -6.0]]
    # single rounding: the exact product 3 * (1+2^-23) * (1+2^-23) is not a float
    s = np.float32(1 + 2.0 ** -23)
    f32, _ = oracle.dequant(np.array([[3]], np.int32), float(s), np.array([s], np.float32))
    exact = 3 * (1 + 2.0 ** -23) ** 2
    assert f32[0, 0] == np.float32(exact)


def test_bf16_rounding_ties_to_even_and_matches_torch():
    acc = np.array([[1, 1, 1, 1]], np.int32)
    scales = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -9, 1 + 2.0 ** -8 + 2.0 ** -20], np.float32)
    _, b16 = oracle.dequant(acc, 1.0, scales)
    assert b16.tolist() == [[0x3F80, 0x3F82, 0x3F80, 0x3F81]]
    rng = np.random.default_rng(3)
    acc = rng.integers(-2 ** 20, 2 ** 20, size=(64, 64)).astype(np.int32)
    scales = (rng.random(64) * 1e-3 + 1e-5).astype(np.float32)
    bias = rng.standard_normal(64).astype(np.float32)
    f32, b16 = oracle.dequant(acc, 0.0123, scales, bias)
    ref = torch.from_numpy(f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b16, ref)


def test_dequant_against_float64_formula_on_config1():
    g, W, Xq, sx = synth.config1_tensors()
    vals, meta, scales = oracle.compress(W, g.N, g.M, g.bits)
    acc = oracle.gemm_sparse(Xq[:16], vals, meta, g.O, g.N, g.M, g.bits)
    f32, _ = oracle.dequant(acc, sx, scales)
    # the dequantised product approximates the fp32 layer on the pruned weights
    Wq = oracle.decompress(vals, meta, g.O, g.K, g.N, g.M, g.bits)
    approx = (Xq[:16].astype(np.float64) * float(sx)) @ (Wq.astype(np.float64) * scales[:, None].astype(np.float64)).T
    assert np.allclose(f32, approx, rtol=1e-6, atol=1e-9)
