"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bars: packed values / indices / scales and int32 accumulators bit-exact; fp32 output within
1e-5 * (|acc| * s_act * s_w + |bias|); bf16 output within one bf16 step of the oracle's rounding.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2206_15014_amd as nm
from paper_2206_15014_amd import synth
from paper_2206_15014_amd.binding import NM_OUT_BF16, NM_OUT_F32, NM_OUT_NONE

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FAST_SCHEMES = [(2, 4, 8), (1, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (2, 8, 8), (1, 8, 8), (1, 8, 4)]
ALL_SCHEMES = FAST_SCHEMES + [(3, 4, 8), (3, 4, 4), (4, 8, 8), (4, 8, 4), (3, 8, 4), (5, 8, 8), (7, 8, 4)]


def say(*a):
    print(*a, flush=True)


def gpu_compress(W, N, M, bits, ldw=None):
    Wt = torch.from_numpy(W).to(DEV)
    if ldw is not None:
        buf = torch.zeros((W.shape[0], ldw), dtype=torch.float32, device=DEV)
        buf[:, :W.shape[1]] = Wt
        Wt = buf[:, :W.shape[1]]
    vals, meta, scales = nm.nm_compress(Wt, N, M, bits)
    torch.cuda.synchronize()
    return vals, meta, scales


def assert_packed_equal(gpu, ref, what):
    for name, g, r in zip(("values", "indices", "scales"), gpu, ref):
        g = g.cpu().numpy()
        assert g.shape == r.shape, (what, name, g.shape, r.shape)
        if not np.array_equal(g, r):
            bad = np.argwhere(g != r)
            raise AssertionError("%s: %s differ at %d places, first %s: gpu %s ref %s"
                                 % (what, name, len(bad), bad[0], g[tuple(bad[0])], r[tuple(bad[0])]))


def bf16_order(bits):
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def check_outputs(acc_ref, sx, scales_ref, bias, acc_gpu=None, f32_gpu=None, bf16_gpu=None, what=""):
    ref_f32, ref_b16 = oracle.dequant(acc_ref, float(sx), scales_ref, bias)
    if acc_gpu is not None:
        assert np.array_equal(acc_gpu, acc_ref), "%s: int32 accumulators differ (%d places)" % (
            what, np.count_nonzero(acc_gpu != acc_ref))
    mag = np.abs(acc_ref).astype(np.float64) * float(sx) * scales_ref[None, :].astype(np.float64)
    if bias is not None:
        mag = mag + np.abs(bias)[None, :].astype(np.float64)
    if f32_gpu is not None:
        err = np.abs(f32_gpu.astype(np.float64) - ref_f32.astype(np.float64))
        assert np.all(err <= 1e-5 * mag + 1e-37), "%s: fp32 output off, worst ratio %g" % (
            what, np.max(err / (mag + 1e-37)))
    if bf16_gpu is not None:
        # One bf16 step from the rounded reference.  Where the bias cancels the product (|y| far
        # below |acc|*s_act*s_w + |bias|) a step of bf16 is smaller than the fp32 tolerance the
        # value was computed to, so there the fp32 band, widened by one bf16 step, decides.
        d = np.abs(bf16_order(bf16_gpu) - bf16_order(ref_b16))
        val = (bf16_gpu.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        band = 1e-5 * mag + np.abs(ref_f32.astype(np.float64)) * 2.0 ** -7 + 1e-37
        ok = (d <= 1) | (np.abs(val - ref_f32.astype(np.float64)) <= band)
        assert np.all(ok), "%s: bf16 output more than one step off at %d places (max %d steps)" % (
            what, np.count_nonzero(~ok), d[~ok].max())


def run_gemm(Xq, sx, packed, O, N, M, bits, bias=None, want=("acc", "f32"), ldo=None):
    vals, meta, scales = packed
    X = torch.from_numpy(Xq).to(DEV)
    T = Xq.shape[0]
    ldo = ldo or O
    b = None if bias is None else torch.from_numpy(bias).to(DEV)
    res = {}
    if "f32" in want or "acc" in want:
        acc = torch.full((T, ldo), -7, dtype=torch.int32, device=DEV) if "acc" in want else None
        out = torch.full((T, ldo), -7.0, dtype=torch.float32, device=DEV) if "f32" in want else None
        nm.nm_gemm(X, float(sx), vals, meta, scales, O, N, M, bits, bias=b, acc=acc, out=out,
                   out_dtype=NM_OUT_F32 if out is not None else NM_OUT_NONE, ldo=ldo)
        torch.cuda.synchronize()
        if acc is not None:
            res["acc"] = acc.cpu().numpy()
        if out is not None:
            res["f32"] = out.cpu().numpy()
    if "bf16" in want:
        out = torch.full((T, ldo), -7.0, dtype=torch.bfloat16, device=DEV)
        nm.nm_gemm(X, float(sx), vals, meta, scales, O, N, M, bits, bias=b, out=out, out_dtype=NM_OUT_BF16, ldo=ldo)
        torch.cuda.synchronize()
        res["bf16"] = out.view(torch.int16).cpu().numpy().view(np.uint16)
    return res


# ---- compress ---------------------------------------------------------------------------------

@pytest.mark.parametrize("N,M,bits", ALL_SCHEMES)
@pytest.mark.parametrize("rows,cols", [(70, 768), (9, 4352), (5, 64), (3, 24), (130, 1024)])
def test_compress_matches_oracle(N, M, bits, rows, cols):
    if cols % M:
        pytest.skip("width not a multiple of M")
    say("compress", N, M, bits, rows, cols)
    rng = np.random.default_rng([N, M, bits, rows, cols])
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    W[rows // 2, : cols // 2] = 0.0
    ref = oracle.compress(W, N, M, bits)
    assert_packed_equal(gpu_compress(W, N, M, bits), ref, "contiguous")
    assert_packed_equal(gpu_compress(W, N, M, bits, ldw=cols + 12), ref, "strided")


@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES + [(3, 4, 8), (4, 8, 4)])
def test_compress_degenerate_rows(N, M, bits):
    say("compress degenerate", N, M, bits)
    for K in (64, 256):
        W = synth.structured_weight_cases(K)
        assert_packed_equal(gpu_compress(W, N, M, bits), oracle.compress(W, N, M, bits), "K=%d" % K)


def test_compress_single_group_rows():
    for N, M, bits in [(2, 4, 8), (1, 4, 4), (2, 8, 4), (1, 8, 8)]:
        W = np.array([[0.5, -1.0, 0.25, 1.0, -0.125, 0.0, 0.75, -0.75][:M]], np.float32)
        assert_packed_equal(gpu_compress(W, N, M, bits), oracle.compress(W, N, M, bits), "K=M")


def test_decompress_round_trip():
    rng = np.random.default_rng(5)
    for N, M, bits in ALL_SCHEMES:
        W = (rng.standard_normal((19, 16 * M)) * 0.02).astype(np.float32)
        vals, meta, _ = oracle.compress(W, N, M, bits)
        out = nm.nm_decompress_i8(torch.from_numpy(vals).to(DEV), torch.from_numpy(meta).to(DEV), 19, 16 * M, N, M, bits)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.decompress(vals, meta, 19, 16 * M, N, M, bits))


# ---- GEMM, small shapes spanning several tiles with ragged edges ------------------------------

def small_case(N, M, bits, T, K, O, seed, with_bias=True):
    rng = np.random.default_rng([N, M, bits, T, K, O, seed])
    W = (rng.standard_normal((O, K)) * 0.02).astype(np.float32)
    Xq, sx = synth.quantize_activations(rng.standard_normal((T, K)).astype(np.float32))
    bias = (rng.standard_normal(O) * 0.02).astype(np.float32) if with_bias else None
    ref = oracle.compress(W, N, M, bits)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
    return W, Xq, sx, bias, ref, acc_ref


@pytest.mark.parametrize("tile", ["0", "1", "2", "3"])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES)
def test_gemm_mfma_path_small(N, M, bits, tile):
    _gemm_small(N, M, bits, tile)


@pytest.mark.parametrize("tile", [str(i) for i in range(4, 18)] + ["101", "105", "109", "112", "113", "115", "116", "117", "119", "121", "122", "128", "201", "202", "203", "204", "205", "206"])
def test_gemm_mfma_path_every_tile_shape(tile):
    _gemm_small(2, 4, 8, tile)


def _gemm_small(N, M, bits, tile):
    say("gemm small", N, M, bits, "tile", tile)
    os.environ["NM_GEMM_TILE"] = tile
    try:
        for T, K, O in [(200, 256, 136), (129, 128, 260), (16, 384, 64), (300, 1408, 200)]:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 1)
            packed = gpu_compress(W, N, M, bits)
            assert_packed_equal(packed, ref, "compress")
            res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32", "bf16"))
            check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], res["bf16"], what="T%d K%d O%d" % (T, K, O))
    finally:
        os.environ.pop("NM_GEMM_TILE", None)


@pytest.mark.parametrize("tile", ["105", "115", "117", "121", "122", "128"])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES[1:])
def test_gemm_decoded_patterns_on_the_large_tiles(N, M, bits, tile):
    """The patterns that are re-encoded in registers, on the tile shapes the launcher picks for
    them on wide and on narrow or long layers: several tiles, ragged edges, K of 2 to 12 slices."""
    say("gemm decoded patterns", N, M, bits, "tile", tile)
    os.environ["NM_GEMM_TILE"] = tile
    try:
        for T, K, O in [(520, 768, 400), (200, 256, 136), (300, 1536, 200)]:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 3)
            packed = gpu_compress(W, N, M, bits)
            res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32", "bf16"))
            check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], res["bf16"], what="T%d K%d O%d" % (T, K, O))
    finally:
        os.environ.pop("NM_GEMM_TILE", None)


STREAM_TILES = ["201", "202", "203", "204", "205", "206"]


@pytest.mark.parametrize("tile", STREAM_TILES)
def test_gemm_persistent_kernel_several_tiles_per_workgroup(tile):
    """Shapes the persistent kernel takes (whole column tiles, dequantised output only): more tiles
    than CUs so that workgroups run on from one tile into the next, one K step per tile, an odd
    number of K steps, a ragged last token tile, and a problem of a single tile."""
    say("gemm persistent tile", tile)
    os.environ["NM_GEMM_TILE"] = tile
    try:
        for T, K, O, with_bias in [(4400, 384, 1536, True), (4400, 128, 1536, False), (100, 256, 384, True), (1, 640, 384, True)]:
            W, Xq, sx, bias, ref, acc_ref = small_case(2, 4, 8, T, K, O, 7, with_bias=with_bias)
            packed = gpu_compress(W, 2, 4, 8)
            f32 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("f32",))["f32"]
            b16 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("bf16",))["bf16"]
            check_outputs(acc_ref, sx, ref[2], bias, None, f32, b16, what="T%d K%d O%d" % (T, K, O))
            if T == 100:     # padded output rows stay untouched
                f32p = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("f32",), ldo=O + 32)["f32"]
                assert np.all(f32p[:, O:] == -7.0)
                check_outputs(acc_ref, sx, ref[2], bias, None, f32p[:, :O], None, what="padded T%d" % T)
    finally:
        os.environ.pop("NM_GEMM_TILE", None)


@pytest.mark.parametrize("tile", ["301", "302"])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (2, 8, 8), (2, 8, 4), (1, 4, 8)])
def test_gemm_x_resident_kernel(N, M, bits, tile):
    """Shapes the X-resident kernel takes (whole 128-token tiles, column tiles in pairs of 192,
    K of 3 to 6 slices, dequantised output only): more workgroups than CUs, every admitted K,
    with and without bias, padded output rows; and shapes it refuses (ragged tokens, odd number
    of column tiles, a pattern with 8-byte stage rows), which must fall through to the other
    kernels with the same results."""
    say("gemm x-resident", N, M, bits, tile)
    os.environ["NM_GEMM_TILE"] = tile
    try:
        cases = [(4480, 768, 1536, True), (256, 384, 768, False), (128, 512, 384, True), (384, 640, 768, True),
                 (100, 768, 768, True), (256, 768, 576, True), (256, 896, 768, True)]
        if (N, M, bits) != (2, 4, 8):
            cases = cases[1:4]
        for T, K, O, with_bias in cases:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 11, with_bias=with_bias)
            packed = gpu_compress(W, N, M, bits)
            f32 = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("f32",))["f32"]
            b16 = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("bf16",))["bf16"]
            check_outputs(acc_ref, sx, ref[2], bias, None, f32, b16, what="T%d K%d O%d" % (T, K, O))
            if T == 256 and K == 384:     # padded output rows stay untouched
                f32p = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("f32",), ldo=O + 32)["f32"]
                assert np.all(f32p[:, O:] == -7.0)
                check_outputs(acc_ref, sx, ref[2], bias, None, f32p[:, :O], None, what="padded T%d" % T)
                b16p = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("bf16",), ldo=O + 32)["bf16"]
                check_outputs(acc_ref, sx, ref[2], bias, None, None, b16p[:, :O], what="padded bf16 T%d" % T)
    finally:
        os.environ.pop("NM_GEMM_TILE", None)


@pytest.mark.parametrize("N,M,bits", ALL_SCHEMES)
def test_gemm_generic_path_odd_shapes(N, M, bits):
    say("gemm generic", N, M, bits)
    for T, K, O in [(1, M, 1), (7, 3 * M, 5), (33, 40, 18), (3, 136, 129)]:
        if K % M:
            continue
        W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 2)
        packed = gpu_compress(W, N, M, bits)
        assert_packed_equal(packed, ref, "compress")
        res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32", "bf16"))
        check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], res["bf16"], what="T%d K%d O%d" % (T, K, O))


def test_gemm_large_output_written_through_with_padded_rows():
    """A bf16 output large enough (>= 14 MB) to take the written-through stores of the wide tile, with
    padded output rows (the padding must stay untouched) and a ragged last column tile."""
    say("gemm large output, padded rows")
    T, K, O = 4096, 256, 2240          # 12 column tiles of 192, the last one 128 wide; 18.4 MB of bf16
    W, Xq, sx, bias, ref, acc_ref = small_case(2, 4, 8, T, K, O, 5)
    packed = gpu_compress(W, 2, 4, 8)
    b16 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("bf16",), ldo=O + 64)["bf16"]
    assert np.all(b16[:, O:] == 0xC0E0)            # -7.0 in bf16: the padding is as the caller left it
    check_outputs(acc_ref, sx, ref[2], bias, None, None, b16[:, :O], what="bf16 through, padded")
    f32 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("f32",), ldo=O + 64)["f32"]
    assert np.all(f32[:, O:] == -7.0)
    check_outputs(acc_ref, sx, ref[2], bias, None, f32[:, :O], None, what="f32 through, padded")


def test_gemm_padded_output_rows_and_no_bias():
    W, Xq, sx, _, ref, acc_ref = small_case(2, 4, 8, 150, 256, 128, 3, with_bias=False)
    packed = gpu_compress(W, 2, 4, 8)
    res = run_gemm(Xq, sx, packed, 128, 2, 4, 8, None, want=("acc", "f32", "bf16"), ldo=160)
    assert np.all(res["acc"][:, 128:] == -7) and np.all(res["f32"][:, 128:] == -7.0)   # padding untouched
    check_outputs(acc_ref, sx, ref[2], None, res["acc"][:, :128], res["f32"][:, :128], res["bf16"][:, :128])


def test_gemm_extreme_codes_do_not_overflow():
    K, O, T = 4096, 16, 16
    W = np.ones((O, K), np.float32)
    Xq = np.full((T, K), -127, np.int8)
    packed = gpu_compress(W, 2, 4, 8)
    res = run_gemm(Xq, 1.0, packed, O, 2, 4, 8, None, want=("acc",))
    assert np.all(res["acc"] == -127 * 127 * (K // 2))


def test_sparse_product_equals_dense_product_on_gpu():
    W, Xq, sx, _, ref, acc_ref = small_case(2, 4, 8, 256, 512, 256, 4, with_bias=False)
    packed = gpu_compress(W, 2, 4, 8)
    Wq = nm.nm_decompress_i8(packed[0], packed[1], 256, 512, 2, 4, 8)
    dense = (torch.from_numpy(Xq).to(DEV).float() @ Wq.float().T).round().to(torch.int32)   # exact: |sum| < 2^24
    res = run_gemm(Xq, sx, packed, 256, 2, 4, 8, None, want=("acc",))
    assert np.array_equal(res["acc"], dense.cpu().numpy())


# ---- the five workloads -----------------------------------------------------------------------

def test_config1_full():
    g, W, Xq, sx = synth.config1_tensors()
    ref = oracle.compress(W, g.N, g.M, g.bits)
    packed = gpu_compress(W, g.N, g.M, g.bits)
    assert_packed_equal(packed, ref, "config 1")
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], g.O, g.N, g.M, g.bits)
    res = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc", "f32", "bf16"))
    check_outputs(acc_ref, sx, ref[2], None, res["acc"], res["f32"], res["bf16"], what="config 1")


def sampled_tokens(T, n=72, seed=0):
    rng = np.random.default_rng(seed)
    edge = np.array([0, 1, 15, 16, 63, 64, 127, 128, T - 129, T - 128, T - 17, T - 2, T - 1])
    return np.unique(np.concatenate([edge[(edge >= 0) & (edge < T)], rng.integers(0, T, size=n)]))


def full_size_case(g):
    """Whole compress compared byte for byte; GEMM compared on sampled token rows, which the
    oracle computes one by one, in the launch configuration the library picks for the full size."""
    say("full size", g)
    W = synth.weights(g)
    Xq, sx = synth.activations(g)
    bias = synth.bias(g)
    ref = oracle.compress(W, g.N, g.M, g.bits)
    packed = gpu_compress(W, g.N, g.M, g.bits)
    assert_packed_equal(packed, ref, g.name)
    rows = sampled_tokens(g.T, seed=g.seed[-1])
    acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
    res = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, bias, want=("acc", "f32", "bf16"))
    check_outputs(acc_ref, sx, ref[2], bias, res["acc"][rows], res["f32"][rows], res["bf16"][rows], what=str(g))
    # every output element was written (the buffers were pre-filled with a sentinel)
    assert not np.any(res["f32"] == -7.0) or np.count_nonzero(res["f32"] == -7.0) < 4


@pytest.mark.parametrize("i", range(4))
def test_config2_bert_base_2of4_int8(i):
    full_size_case(synth.config2()[i])


@pytest.mark.parametrize("i", range(4))
def test_config3_bert_large_2of4_int8(i):
    full_size_case(synth.config3()[i])


@pytest.mark.parametrize("i", range(8))
def test_config4_int4_1of4_and_2of8(i):
    full_size_case(synth.config4()[i])


def test_config5_heterogeneous_encoder_back_to_back():
    gs = synth.config5()
    say("config 5 schemes", [(g.N, g.M, g.bits) for g in gs])
    # one X per distinct reduction width (768 / 3072) keeps host memory and time small; weights differ per GEMM
    acts = {}
    for g in gs:
        if g.K not in acts:
            acts[g.K] = synth.activations(g)
    stream = torch.cuda.current_stream()
    jobs = []
    for g in gs:
        W = synth.weights(g)
        ref = oracle.compress(W, g.N, g.M, g.bits)
        packed = nm.nm_compress(torch.from_numpy(W).to(DEV), g.N, g.M, g.bits)
        Xq, sx = acts[g.K]
        X = torch.from_numpy(Xq).to(DEV)
        acc = torch.empty((g.T, g.O), dtype=torch.int32, device=DEV)
        out = torch.empty((g.T, g.O), dtype=torch.bfloat16, device=DEV)
        jobs.append((g, ref, packed, X, sx, acc, out))
    torch.cuda.synchronize()
    for g, ref, packed, X, sx, acc, out in jobs:          # all 48 launches back to back on one stream
        nm.nm_gemm(X, float(sx), *packed, g.O, g.N, g.M, g.bits, acc=acc, out=out, out_dtype=NM_OUT_BF16, stream=stream)
    torch.cuda.synchronize()
    for g, ref, packed, X, sx, acc, out in jobs:
        assert_packed_equal(packed, ref, str(g))
        rows = sampled_tokens(g.T, n=24, seed=g.seed[1] * 4 + g.seed[2])
        Xq = acts[g.K][0]
        acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
        check_outputs(acc_ref, sx, ref[2], None, acc.cpu().numpy()[rows], None,
                      out.view(torch.int16).cpu().numpy().view(np.uint16)[rows], what=str(g))


def test_results_do_not_depend_on_repetition():
    g = synth.config2()[3]
    W, (Xq, sx) = synth.weights(g), synth.activations(g)
    packed = gpu_compress(W, g.N, g.M, g.bits)
    a = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",))["acc"]
    b = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",))["acc"]
    assert np.array_equal(a, b)


# ---- requantised output (nm_gemm_q8): codes and max |y| bit-exact -------------------------------
def run_gemm_q8(Xq, sx, packed, O, N, M, bits, bias, out_scale, ldo=None, start_max=0.0):
    vals, meta, scales = packed
    X = torch.from_numpy(Xq).to(DEV)
    T = Xq.shape[0]
    ldo = ldo or O
    b = None if bias is None else torch.from_numpy(bias).to(DEV)
    out = torch.full((T, ldo), -77, dtype=torch.int8, device=DEV)
    amax = torch.full((1,), start_max, dtype=torch.float32, device=DEV)
    nm.nm_gemm_q8(X, float(sx), vals, meta, scales, O, N, M, bits, float(out_scale), out, bias=b, absmax=amax, ldo=ldo)
    torch.cuda.synchronize()
    return out.cpu().numpy(), float(amax.item())


def check_q8(acc_ref, sx, scales_ref, bias, out_scale, q_gpu, amax_gpu, what=""):
    q_ref, amax_ref = oracle.requant(acc_ref, float(sx), scales_ref, float(out_scale), bias)
    assert np.array_equal(q_gpu, q_ref), "%s: int8 codes differ at %d places" % (what, np.count_nonzero(q_gpu != q_ref))
    assert amax_gpu == amax_ref, "%s: max |y| %r against %r" % (what, amax_gpu, amax_ref)


def q8_scale(acc_ref, sx, scales_ref, bias):
    """An output scale that uses the code range: max |y| / 127, as a caller would choose it."""
    f32, _ = oracle.dequant(acc_ref, float(sx), scales_ref, bias)
    return np.float32(np.abs(f32).max() / 127.0)


@pytest.mark.parametrize("tile", ["0", "2", "113", "116", "122", "201", "301"])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 4, 4), (2, 8, 4)])
def test_gemm_q8_fast_paths(N, M, bits, tile):
    """Every kernel family (201 and 301 do not write codes and must hand the call on), whole and
    ragged tiles, rows of 16-byte, 8-byte and 4-byte granularity, with and without bias."""
    say("gemm q8", N, M, bits, "tile", tile)
    os.environ["NM_GEMM_TILE"] = tile
    try:
        for T, K, O, with_bias, pad in [(300, 256, 392, True, 0), (129, 512, 260, False, 0), (512, 768, 768, True, 8), (16, 384, 64, True, 4), (300, 256, 384, True, 16)]:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 21, with_bias=with_bias)
            packed = gpu_compress(W, N, M, bits)
            so = q8_scale(acc_ref, sx, ref[2], bias)
            q, amax = run_gemm_q8(Xq, sx, packed, O, N, M, bits, bias, so, ldo=O + pad)
            assert np.all(q[:, O:] == -77)                 # padding untouched
            check_q8(acc_ref, sx, ref[2], bias, so, q[:, :O], amax, what="T%d K%d O%d" % (T, K, O))
    finally:
        os.environ.pop("NM_GEMM_TILE", None)


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (3, 4, 8), (4, 8, 4), (1, 8, 8)])
def test_gemm_q8_generic_path_and_saturation(N, M, bits):
    say("gemm q8 generic", N, M, bits)
    for T, K, O in [(7, 3 * M, 5), (33, 40, 18), (3, 136, 129)]:
        if K % M:
            continue
        W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 22)
        packed = gpu_compress(W, N, M, bits)
        so = q8_scale(acc_ref, sx, ref[2], bias)
        for scale in (so, np.float32(so / 16)):            # the second one saturates most codes at +-127
            q, amax = run_gemm_q8(Xq, sx, packed, O, N, M, bits, bias, scale)
            check_q8(acc_ref, sx, ref[2], bias, scale, q, amax, what="T%d K%d O%d scale %g" % (T, K, O, scale))
            assert q.min() >= -127


def test_gemm_q8_running_maximum_is_kept():
    W, Xq, sx, bias, ref, acc_ref = small_case(2, 4, 8, 64, 256, 96, 23)
    packed = gpu_compress(W, 2, 4, 8)
    so = q8_scale(acc_ref, sx, ref[2], bias)
    _, amax_ref = oracle.requant(acc_ref, float(sx), ref[2], float(so), bias)
    _, amax = run_gemm_q8(Xq, sx, packed, 96, 2, 4, 8, bias, so, start_max=amax_ref * 4.0)
    assert amax == np.float32(amax_ref * 4.0)              # a larger value already there survives
    _, amax = run_gemm_q8(Xq, sx, packed, 96, 2, 4, 8, bias, so, start_max=amax_ref / 4.0)
    assert amax == amax_ref


def test_gemm_q8_full_size_layer_feeds_the_next_one():
    """BERT-base FFN-up at 4096 tokens in the configuration the benchmark uses, its codes checked in
    full, then used as the activations of FFN-down: the chain never leaves int8."""
    say("gemm q8 full size")
    g_up, g_down = [g for g in synth.config2() if g.name in ("ffn_up", "ffn_down")]
    W = synth.weights(g_up); Xq, sx = synth.activations(g_up); bias = synth.bias(g_up)
    ref = oracle.compress(W, 2, 4, 8)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], g_up.O, 2, 4, 8)
    packed = gpu_compress(W, 2, 4, 8)
    so = q8_scale(acc_ref, sx, ref[2], bias)
    q, amax = run_gemm_q8(Xq, sx, packed, g_up.O, 2, 4, 8, bias, so)
    check_q8(acc_ref, sx, ref[2], bias, so, q, amax, what="ffn_up")
    W2 = synth.weights(g_down)
    ref2 = oracle.compress(W2, 2, 4, 8)
    acc2_ref = oracle.gemm_sparse(q, ref2[0], ref2[1], g_down.O, 2, 4, 8)
    packed2 = gpu_compress(W2, 2, 4, 8)
    res = run_gemm(q, so, packed2, g_down.O, 2, 4, 8, None, want=("acc",))
    assert np.array_equal(res["acc"], acc2_ref)


# ---- ADMM Z-update (nm_project): Z, the dual update and the scales bit-exact ---------------------
def run_project(W, U, N, M, bits, rps, pad=0, in_place=False):
    rows, cols = W.shape
    ld = cols + pad
    Wd = torch.zeros((rows, ld), dtype=torch.float32, device=DEV)
    Wd[:, :cols] = torch.from_numpy(W).to(DEV)
    Ud = None
    if U is not None:
        Ud = torch.zeros((rows, ld), dtype=torch.float32, device=DEV)
        Ud[:, :cols] = torch.from_numpy(U).to(DEV)
    Z = torch.full((rows, ld), -7.0, dtype=torch.float32, device=DEV)
    Uo = Ud if in_place else torch.full((rows, ld), -7.0, dtype=torch.float32, device=DEV)
    Zv, Uov, scales = nm.nm_project(Wd[:, :cols], None if Ud is None else Ud[:, :cols], N, M, bits, rps,
                                    Z=Z[:, :cols], U_out=Uo[:, :cols])
    torch.cuda.synchronize()
    return Z.cpu().numpy(), Uo.cpu().numpy(), None if scales is None else scales.cpu().numpy()


@pytest.mark.parametrize("rps", [1, 32, 1000])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 8), (3, 4, 0), (2, 8, 4), (4, 8, 8), (1, 8, 0), (2, 4, 0)])
def test_project_matches_oracle(N, M, bits, rps):
    say("project", N, M, bits, "rows per scale", rps)
    rng = np.random.default_rng([N, M, bits, rps])
    for rows, cols, with_u, pad in [(70, 24 * M, True, 0), (257, 96, False, 4), (5, M, True, 8), (768, 768, True, 0)]:
        W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
        W[rng.integers(0, rows), :] = 0.0                                   # a zero row
        W[:, : 2 * M] = np.round(W[:, : 2 * M] * 64) / 64                   # ties inside groups
        U = (rng.standard_normal((rows, cols)) * 0.004).astype(np.float32) if with_u else None
        Zr, Ur, sr = oracle.admm_project(W, U, N, M, bits, rps)
        Z, Uo, s = run_project(W, U, N, M, bits, rps, pad=pad)
        what = "rows %d cols %d" % (rows, cols)
        assert np.array_equal(Z[:, :cols].view(np.uint32), Zr.view(np.uint32)), what + ": Z differs"   # signed zeros too
        assert np.array_equal(Uo[:, :cols].view(np.uint32), Ur.view(np.uint32)), what + ": U differs"
        if pad:
            assert np.all(Z[:, cols:] == -7.0) and np.all(Uo[:, cols:] == -7.0)
        if bits:
            assert np.array_equal(s, sr), what + ": scales differ"
        else:
            assert s is None


def test_project_dual_update_in_place_and_full_size():
    """BERT-base FFN-up weights with the paper's default scale groups (32 neurons); U updated in place."""
    say("project full size")
    g = [g for g in synth.config2() if g.name == "ffn_up"][0]
    W = synth.weights(g)
    rng = np.random.default_rng(9)
    U = (rng.standard_normal(W.shape) * 0.002).astype(np.float32)
    Zr, Ur, sr = oracle.admm_project(W, U, 2, 4, 8, 32)
    Z, Uo, s = run_project(W, U, 2, 4, 8, 32, in_place=True)
    assert np.array_equal(Z.view(np.uint32), Zr.view(np.uint32))
    assert np.array_equal(Uo.view(np.uint32), Ur.view(np.uint32))
    assert np.array_equal(s, sr)
    # what the projection is for: Z satisfies both constraints
    assert np.all(np.count_nonzero(Z.reshape(W.shape[0], -1, 4), axis=2) <= 2)
    codes = Z / s[:, None]
    assert np.all(np.abs(codes - np.rint(codes)) < 1e-3) and np.abs(np.rint(codes)).max() == 127


# ---- one scale per group of rows (nm_compress_grouped): packed bytes and scales bit-exact --------
@pytest.mark.parametrize("rps", [2, 32, 100])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES + [(3, 4, 8), (4, 8, 4)])
def test_compress_grouped_matches_oracle_and_feeds_the_gemm(N, M, bits, rps):
    say("compress grouped", N, M, bits, "rows per scale", rps)
    rng = np.random.default_rng([N, M, bits, rps, 3])
    for rows, cols, ldw in [(70, 256, None), (257, 1408, None), (768, 768, 776), (5, 8 * M, None), (33, 40, None)]:
        if cols % M:
            continue
        W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
        W[rng.integers(0, rows)] = 0.0
        ref = oracle.compress_grouped(W, N, M, bits, rps)
        Wt = torch.from_numpy(W).to(DEV)
        if ldw is not None:
            buf = torch.zeros((rows, ldw), dtype=torch.float32, device=DEV)
            buf[:, :cols] = Wt
            Wt = buf[:, :cols]
        packed = nm.nm_compress_grouped(Wt, N, M, bits, rps)
        torch.cuda.synchronize()
        assert_packed_equal(packed, ref, "grouped %dx%d" % (rows, cols))
    # the packed result is an ordinary operand of nm_gemm
    T, K, O = 200, 256, 136
    W, Xq, sx, bias, _, _ = small_case(N, M, bits, T, K, O, 4)
    ref = oracle.compress_grouped(W, N, M, bits, rps)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
    packed = nm.nm_compress_grouped(torch.from_numpy(W).to(DEV), N, M, bits, rps)
    res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32"))
    check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], None, what="gemm on grouped scales")


# ---- several matrices in one call (nm_compress_batch): byte for byte what nm_compress gives -----
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 4, 4), (2, 8, 4), (4, 8, 8), (3, 4, 8)])
def test_compress_batch_matches_oracle_item_by_item(N, M, bits):
    """Matrices of different heights and widths in one call: one, two and four wavefronts per row
    (widths up to 3072), a height that is not a multiple of the rows per workgroup, a padded
    leading dimension, a matrix whose packed rows are not whole dwords (goes out on its own), more
    matrices than one launch takes (17 of them follow), and 3:4, which no wavefront kernel covers."""
    say("compress batch", N, M, bits)
    rng = np.random.default_rng([N, M, bits, 77])
    shapes = [(37, 768, 768), (5, 3072, 3072), (130, 1536, 1600), (9, 5 * M, 5 * M), (64, 256, 256)] + [(3 + i, 128, 128) for i in range(17)]
    Ws, dev = [], []
    for rows, cols, ldw in shapes:
        W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
        W[rows // 2, :] = 0.0                                  # an all-zero row: scale 1
        buf = torch.zeros((rows, ldw), dtype=torch.float32, device=DEV)
        buf[:, :cols] = torch.from_numpy(W).to(DEV)
        Ws.append(W)
        dev.append(buf[:, :cols])
    outs = nm.nm_compress_batch(dev, N, M, bits)
    torch.cuda.synchronize()
    for W, packed, shape in zip(Ws, outs, shapes):
        assert_packed_equal(packed, oracle.compress(W, N, M, bits), "batch item %s" % (shape,))


def test_compress_batch_full_size_layer_set_feeds_the_gemm():
    gs = synth.config2()
    Ws = [synth.weights(g) for g in gs]
    outs = nm.nm_compress_batch([torch.from_numpy(W).to(DEV) for W in Ws], 2, 4, 8)
    torch.cuda.synchronize()
    for g, W, packed in zip(gs, Ws, outs):
        ref = oracle.compress(W, g.N, g.M, g.bits)
        assert_packed_equal(packed, ref, "batch " + g.name)
    g, W, packed = gs[1], Ws[1], outs[1]
    Xq, sx = synth.activations(g)
    rows = sampled_tokens(g.T, n=16, seed=5)
    ref = oracle.compress(W, g.N, g.M, g.bits)
    acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
    acc = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",))["acc"]
    assert np.array_equal(acc[rows], acc_ref)


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 8), (2, 8, 4)])
def test_compress_quotients_next_to_half_way_points(N, M, bits):
    """Weights placed on and a few units in the last place around (k + 1/2) * scale, for scales
    with arbitrary significands (all ones and all zeros among them) over the exponent range,
    including scales outside the range in which the kernel divides by way of the reciprocal: the
    codes hinge on the correctly rounded quotient, which the oracle takes from the division operator."""
    say("compress half-way quotients", N, M, bits)
    rng = np.random.default_rng([N, M, bits, 5])
    qmax = (1 << (bits - 1)) - 1
    rows, cols = 96, 64 * M
    W = np.zeros((rows, cols), np.float32)
    for r in range(rows):
        mant = [0, (1 << 23) - 1, 1, (1 << 23) - 2][r % 8] if r % 8 < 4 else int(rng.integers(0, 1 << 23))
        expo = 127 + [-70, -61, -60, -30, -8, 0, 9, 31, 59, 60, 61, 70][r % 12]
        amax = np.array([(expo << 23) | mant], np.uint32).view(np.float32)[0]
        scale = np.float32(amax) / np.float32(qmax)                      # what the row's scale will be
        k = rng.integers(-qmax, qmax, cols).astype(np.float64) + 0.5
        w = (k * np.float64(scale)).astype(np.float32)
        w = (w.view(np.int32) + rng.integers(-2, 3, cols).astype(np.int32)).view(np.float32)
        w = np.clip(w, -amax, amax)
        w[int(rng.integers(0, cols))] = amax
        W[r] = w
    assert np.isfinite(W).all()
    packed = gpu_compress(W, N, M, bits)
    assert_packed_equal(packed, oracle.compress(W, N, M, bits), "half-way quotients")


def test_compress_batch_and_gemm_replayed_from_a_graph():
    """The launches as bench.py issues them: nm_compress_batch and nm_gemm captured once in a HIP
    graph and replayed, the weights changed in place between the replays (and eager work and
    synchronisations in between); every replay must give what the oracle gives for the weights
    of that moment."""
    say("graph replay: compress batch + gemm")
    N, M, bits = 2, 4, 8
    rng = np.random.default_rng(99)
    shapes = [(96, 256), (40, 768)]
    Ws = [(rng.standard_normal(sh) * 0.02).astype(np.float32) for sh in shapes]
    Wd = [torch.from_numpy(W).to(DEV) for W in Ws]
    outs = nm.nm_compress_batch(Wd, N, M, bits)             # allocates the packed buffers (and warms up)
    T, K, O = 200, 256, 96
    Xq, sx = synth.quantize_activations(rng.standard_normal((T, K)).astype(np.float32))
    X = torch.from_numpy(Xq).to(DEV)
    acc = torch.empty((T, O), dtype=torch.int32, device=DEV)
    y = torch.empty((T, O), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        nm.nm_gemm(X, float(sx), *outs[0], O, N, M, bits, acc=acc, out=y, out_dtype=NM_OUT_F32, stream=side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            nm.nm_compress_batch(Wd, N, M, bits, outs=outs, stream=side)
            nm.nm_gemm(X, float(sx), *outs[0], O, N, M, bits, acc=acc, out=y, out_dtype=NM_OUT_F32, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for W, d in zip(Ws, Wd):                            # new weights in the same buffers
            W[...] = (rng.standard_normal(W.shape) * 0.02 * (rep + 1)).astype(np.float32)
            d.copy_(torch.from_numpy(W))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for W, packed in zip(Ws, outs):
            assert_packed_equal(packed, oracle.compress(W, N, M, bits), "replay %d" % rep)
        ref = oracle.compress(Ws[0], N, M, bits)
        acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
        check_outputs(acc_ref, sx, ref[2], None, acc.cpu().numpy(), y.cpu().numpy(), None, what="replay %d" % rep)
