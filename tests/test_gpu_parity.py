"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bars: packed values / indices / scales and int32 accumulators bit-exact, in both layouts of the
packed buffers; fp32 output within 1e-5 * (|acc| * s_act * s_w + |bias|); bf16 output within one
bf16 step of the oracle's rounding; int8 output codes equal to the oracle's except within a
stated distance of a half-way point (see check_q8).
"""
import contextlib

import numpy as np
import pytest
import torch

import oracle
import paper_2206_15014_amd as nm
from paper_2206_15014_amd import binding, synth
from paper_2206_15014_amd.binding import NM_LAYOUT_ROWS as ROWS, NM_LAYOUT_TILED as TILED, NM_OUT_BF16, NM_OUT_F32, NM_OUT_NONE

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FAST_SCHEMES = [(2, 4, 8), (1, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (2, 8, 8), (1, 8, 8), (1, 8, 4)]
DUAL_SCHEMES = [(3, 4, 8), (3, 4, 4), (4, 8, 8), (4, 8, 4), (4, 4, 8), (4, 4, 4)]      # two operands per unit on the matrix pipe
ALL_SCHEMES = FAST_SCHEMES + DUAL_SCHEMES + [(3, 8, 4), (5, 8, 8), (7, 8, 4), (8, 8, 8), (8, 8, 4)]
LAYOUTS = [ROWS, TILED]
# tile variants of the LDS-direct kernels (tiled layout); the second list is what the two-operand patterns compile
DMA_TILES = [112, 113, 115, 116, 117, 121, 122, 123, 128, 130, 132, 133, 136]
DUAL_TILES = [112, 115, 116, 117]
ODD8_SCHEMES = [(n, 8, b) for n in (3, 5, 6, 7) for b in (8, 4)]     # units of 6 .. 28 bytes, also two operands per unit
ODD8_TILES = [115, 116, 117, 127]


def say(*a):
    print(*a, flush=True)


@contextlib.contextmanager
def forced_tile(cfg):
    """Force a tile variant of nm_gemm for the duration of the block (test hook of the library)."""
    binding.force_gemm_tile(int(cfg))
    try:
        yield
    finally:
        binding.force_gemm_tile(0)


def oracle_packed(W, N, M, bits, layout=ROWS, rows_per_scale=1):
    """(vals, meta, scales) as the oracle packs them, in the given layout (tiled: flat byte arrays)."""
    vals, meta, scales = oracle.compress_grouped(W, N, M, bits, rows_per_scale)
    if layout == TILED:
        vals, meta = oracle.to_tiled(vals, meta, W.shape[1], N, M, bits)
    return vals, meta, scales


def gpu_compress(W, N, M, bits, ldw=None, layout=ROWS):
    Wt = torch.from_numpy(W).to(DEV)
    if ldw is not None:
        buf = torch.zeros((W.shape[0], ldw), dtype=torch.float32, device=DEV)
        buf[:, :W.shape[1]] = Wt
        Wt = buf[:, :W.shape[1]]
    rows, cols = W.shape
    vb, mb, _ = nm.nm_packed_sizes(rows, cols, N, M, bits, layout)
    # pre-filled: bytes the kernel leaves out (padding rows of the tiled layout) would show
    shape = (lambda n: (rows, n // rows)) if layout == ROWS else (lambda n: (n,))
    vals = torch.full(shape(vb), 0xA5, dtype=torch.uint8, device=DEV)
    meta = torch.full(shape(mb), 0xA5, dtype=torch.uint8, device=DEV)
    vals, meta, scales = nm.nm_compress(Wt, N, M, bits, vals=vals, meta=meta, layout=layout)
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
        # One bf16 step from the rounded reference, everywhere.  The only exception: where the bias
        # cancels the product so far that the fp32 tolerance the value is computed to (1e-5 of the
        # magnitudes that went in) is itself more than half a bf16 step of the reference; there
        # the fp32 band decides, widened by that one step.  A step is taken from the reference's
        # exponent: 2^(floor(log2 |ref|) - 7).
        d = np.abs(bf16_order(bf16_gpu) - bf16_order(ref_b16))
        ref64 = ref_f32.astype(np.float64)
        step = np.where(ref64 != 0, 2.0 ** (np.floor(np.log2(np.abs(ref64) + (ref64 == 0))) - 7), 0.0)
        cancelled = 1e-5 * mag > 0.5 * step
        val = (bf16_gpu.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        ok = (d <= 1) | (cancelled & (np.abs(val - ref64) <= 1e-5 * mag + step + 1e-37))
        assert np.all(ok), "%s: bf16 output more than one step off at %d places (max %d steps)" % (
            what, np.count_nonzero(~ok), d[~ok].max())
        assert np.count_nonzero(cancelled) <= 4e-3 * cancelled.size + 2, "%s: the cancellation band covers %d outputs" % (
            what, np.count_nonzero(cancelled))


def run_gemm(Xq, sx, packed, O, N, M, bits, bias=None, want=("acc", "f32"), ldo=None, layout=ROWS):
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
                   out_dtype=NM_OUT_F32 if out is not None else NM_OUT_NONE, ldo=ldo, layout=layout)
        torch.cuda.synchronize()
        if acc is not None:
            res["acc"] = acc.cpu().numpy()
        if out is not None:
            res["f32"] = out.cpu().numpy()
    if "bf16" in want:
        out = torch.full((T, ldo), -7.0, dtype=torch.bfloat16, device=DEV)
        nm.nm_gemm(X, float(sx), vals, meta, scales, O, N, M, bits, bias=b, out=out, out_dtype=NM_OUT_BF16, ldo=ldo, layout=layout)
        torch.cuda.synchronize()
        res["bf16"] = out.view(torch.int16).cpu().numpy().view(np.uint16)
    if "f32only" in want:                       # dequantised output alone: the kernels' fast fp32 epilogue
        out = torch.full((T, ldo), -7.0, dtype=torch.float32, device=DEV)
        nm.nm_gemm(X, float(sx), vals, meta, scales, O, N, M, bits, bias=b, out=out, out_dtype=NM_OUT_F32, ldo=ldo, layout=layout)
        torch.cuda.synchronize()
        res["f32only"] = out.cpu().numpy()
    return res


# ---- compress ---------------------------------------------------------------------------------

@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("N,M,bits", ALL_SCHEMES + [(3, 8, 8), (5, 8, 4), (6, 8, 8), (6, 8, 4), (7, 8, 8)])
@pytest.mark.parametrize("rows,cols", [(70, 768), (9, 4352), (5, 64), (3, 24), (130, 1024)])
def test_compress_matches_oracle(N, M, bits, rows, cols, layout):
    if cols % M or (layout == TILED and cols % 128):
        pytest.skip("width not a multiple of M (tiled layout: of 128)")
    say("compress", N, M, bits, rows, cols, "layout", layout)
    rng = np.random.default_rng([N, M, bits, rows, cols])
    W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    W[rows // 2, : cols // 2] = 0.0
    ref = oracle_packed(W, N, M, bits, layout)
    assert_packed_equal(gpu_compress(W, N, M, bits, layout=layout), ref, "contiguous")
    assert_packed_equal(gpu_compress(W, N, M, bits, ldw=cols + 12, layout=layout), ref, "strided")


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES + [(3, 4, 8), (4, 8, 4), (4, 4, 8), (8, 8, 4)])
def test_compress_degenerate_rows(N, M, bits, layout):
    say("compress degenerate", N, M, bits, "layout", layout)
    for K in (64, 256):
        if layout == TILED and K % 128:
            continue
        W = synth.structured_weight_cases(K)
        assert_packed_equal(gpu_compress(W, N, M, bits, layout=layout), oracle_packed(W, N, M, bits, layout), "K=%d" % K)


def test_compress_single_group_rows():
    for N, M, bits in [(2, 4, 8), (1, 4, 4), (2, 8, 4), (1, 8, 8), (4, 4, 8)]:
        W = np.array([[0.5, -1.0, 0.25, 1.0, -0.125, 0.0, 0.75, -0.75][:M]], np.float32)
        assert_packed_equal(gpu_compress(W, N, M, bits), oracle.compress(W, N, M, bits), "K=M")


@pytest.mark.parametrize("layout", LAYOUTS)
def test_decompress_round_trip(layout):
    rng = np.random.default_rng(5)
    for N, M, bits in ALL_SCHEMES:
        W = (rng.standard_normal((19, 128)) * 0.02).astype(np.float32)
        vals, meta, _ = oracle.compress(W, N, M, bits)
        want = oracle.decompress(vals, meta, 19, 128, N, M, bits)
        if layout == TILED:
            vals, meta = oracle.to_tiled(vals, meta, 128, N, M, bits)
        m = torch.from_numpy(meta).to(DEV) if meta.size else None
        out = nm.nm_decompress_i8(torch.from_numpy(vals).to(DEV), m, 19, 128, N, M, bits, layout=layout)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want), (N, M, bits)


@pytest.mark.parametrize("N,M,bits", ALL_SCHEMES)
def test_repack_between_the_layouts(N, M, bits):
    rng = np.random.default_rng([N, M, bits, 44])
    for rows, cols in [(37, 256), (768, 768), (5, 128)]:
        W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
        vr, mr, _ = oracle.compress(W, N, M, bits)
        vt, mt = oracle.to_tiled(vr, mr, cols, N, M, bits)
        dv, dm = torch.from_numpy(vr).to(DEV), torch.from_numpy(mr).to(DEV)
        v2, m2 = nm.nm_repack(dv, dm, rows, cols, N, M, bits, ROWS)
        torch.cuda.synchronize()
        assert np.array_equal(v2.cpu().numpy(), vt) and np.array_equal(m2.cpu().numpy(), mt)
        v3, m3 = nm.nm_repack(v2, m2, rows, cols, N, M, bits, TILED)
        torch.cuda.synchronize()
        assert np.array_equal(v3.cpu().numpy(), vr) and np.array_equal(m3.cpu().numpy(), mr)


# ---- GEMM, small shapes spanning several tiles with ragged edges ------------------------------

def small_case(N, M, bits, T, K, O, seed, with_bias=True):
    rng = np.random.default_rng([N, M, bits, T, K, O, seed])
    W = (rng.standard_normal((O, K)) * 0.02).astype(np.float32)
    Xq, sx = synth.quantize_activations(rng.standard_normal((T, K)).astype(np.float32))
    bias = (rng.standard_normal(O) * 0.02).astype(np.float32) if with_bias else None
    ref = oracle.compress(W, N, M, bits)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
    return W, Xq, sx, bias, ref, acc_ref


SMALL_SHAPES = [(200, 256, 136), (129, 128, 260), (16, 384, 64), (300, 1408, 200)]


def _gemm_small(N, M, bits, tile, layout, shapes=SMALL_SHAPES, seed=1):
    say("gemm small", N, M, bits, "tile", tile, "layout", layout)
    with forced_tile(tile):
        for T, K, O in shapes:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, seed)
            packed = gpu_compress(W, N, M, bits, layout=layout)
            assert_packed_equal(packed, oracle_packed(W, N, M, bits, layout), "compress")
            res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32", "bf16", "f32only"), layout=layout)
            check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], res["bf16"], what="T%d K%d O%d" % (T, K, O))
            check_outputs(acc_ref, sx, ref[2], bias, None, res["f32only"], None, what="f32 alone T%d K%d O%d" % (T, K, O))


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES)
def test_gemm_row_layout_register_staged_kernel(N, M, bits, tile):
    _gemm_small(N, M, bits, tile, ROWS)


@pytest.mark.parametrize("tile", [0] + DMA_TILES)
def test_gemm_tiled_layout_every_tile_shape(tile):
    _gemm_small(2, 4, 8, tile, TILED)


@pytest.mark.parametrize("tile", [0, 113, 115, 117, 121, 122, 127, 128, 130, 132, 133])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES[1:])
def test_gemm_decoded_patterns_on_the_tiled_kernels(N, M, bits, tile):
    """The patterns that are re-encoded in registers, on the tile shapes the launcher picks for
    them on wide and on narrow or long layers: several tiles, ragged edges, K of 2 to 12 slices."""
    _gemm_small(N, M, bits, tile, TILED, shapes=[(520, 768, 400), (200, 256, 136), (300, 1536, 200)], seed=3)


@pytest.mark.parametrize("tile", [0] + DUAL_TILES + [121, 122, 126, 127, 128, 133])
@pytest.mark.parametrize("N,M,bits", DUAL_SCHEMES + [(8, 8, 8)])
def test_gemm_two_operand_patterns_on_the_matrix_pipe(N, M, bits, tile):
    """3:4, 4:8 and dense matrices (more than two kept entries per subgroup of four): each unit is
    multiplied as two operands of the sparse MFMA.  Ragged tiles, K of 1 to 11 slices, a row count
    that is not a multiple of 16 (the tiled layout's padding rows are read, as zeros)."""
    _gemm_small(N, M, bits, tile, TILED, shapes=[(200, 256, 136), (129, 128, 260), (300, 1408, 200), (520, 768, 404)], seed=4)


@pytest.mark.parametrize("tile", [0] + ODD8_TILES)
@pytest.mark.parametrize("N,M,bits", ODD8_SCHEMES)
def test_gemm_other_patterns_of_eight_on_the_matrix_pipe(N, M, bits, tile):
    """3:8, 5:8, 6:8 and 7:8: the kept entries of a group are scattered to their columns in registers and
    the group is multiplied as two operands of the sparse MFMA, like a dense one.  Units of 6 to 28 bytes
    (pieces of 2, 4 or 8 bytes in the tiled layout), ragged tiles, K of 1 to 11 slices."""
    _gemm_small(N, M, bits, tile, TILED, shapes=[(200, 256, 136), (129, 128, 260), (300, 1408, 200), (520, 768, 404)], seed=6)


def _gemm_batch(N, M, bits, layout, tile, shapes, seed, shared_x=False):
    """nm_gemm_batch over `shapes` [(T, K, O), ...] against the oracle item by item: accumulators + fp32 in
    one call, bf16 in another (the kernels' epilogues); outputs padded, the padding must stay as it was."""
    say("gemm batch", N, M, bits, "layout", layout, "tile", tile, shapes)
    cases = [small_case(N, M, bits, T, K, O, seed + i) for i, (T, K, O) in enumerate(shapes)]
    if shared_x:                              # query, key and value: one activation tensor
        cases = [(c[0], cases[0][1], cases[0][2], c[3], c[4],
                  oracle.gemm_sparse(cases[0][1], c[4][0], c[4][1], shapes[i][2], N, M, bits)) for i, c in enumerate(cases)]
    X0 = torch.from_numpy(cases[0][1]).to(DEV)
    with forced_tile(tile):
        for dtype, code in ((torch.float32, NM_OUT_F32), (torch.bfloat16, NM_OUT_BF16)):
            calls, keep = [], []
            for (T, K, O), (W, Xq, sx, bias, ref, acc_ref) in zip(shapes, cases):
                packed = gpu_compress(W, N, M, bits, layout=layout)
                ldo = O + 8
                acc = torch.full((T, ldo), -7, dtype=torch.int32, device=DEV) if code == NM_OUT_F32 else None
                out = torch.full((T, ldo), -7.0, dtype=dtype, device=DEV)
                calls.append(dict(X=X0 if shared_x else torch.from_numpy(Xq).to(DEV), act_scale=float(sx), vals=packed[0], meta=packed[1],
                                  scales=packed[2], O=O, bias=torch.from_numpy(bias).to(DEV), acc=acc, out=out, ldo=ldo))
                keep.append((acc, out))
            nm.nm_gemm_batch(calls, N, M, bits, out_dtype=code, layout=layout)
            torch.cuda.synchronize()
            for i, ((T, K, O), (W, Xq, sx, bias, ref, acc_ref), (acc, out)) in enumerate(zip(shapes, cases, keep)):
                what = "item %d T%d K%d O%d" % (i, T, K, O)
                if code == NM_OUT_F32:
                    a, f = acc.cpu().numpy(), out.cpu().numpy()
                    assert np.all(a[:, O:] == -7) and np.all(f[:, O:] == -7.0), what + ": padding touched"
                    check_outputs(acc_ref, sx, ref[2], bias, a[:, :O], f[:, :O], None, what=what)
                else:
                    b16 = out.view(torch.int16).cpu().numpy().view(np.uint16)
                    assert np.all(b16[:, O:] == 0xC0E0), what + ": padding touched"
                    check_outputs(acc_ref, sx, ref[2], bias, None, None, b16[:, :O], what=what)


@pytest.mark.parametrize("tile", [0, 116, 122, 130, 133])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 8, 8), (4, 4, 4), (4, 8, 8), (3, 4, 8)])
def test_gemm_batch_one_launch_for_several_layers(N, M, bits, tile):
    """Items of different shapes (ragged tiles, K of 1 to 6 slices) whose tiles share one launch of a
    tiled-layout kernel; then query / key / value: three layers on one activation tensor."""
    _gemm_batch(N, M, bits, TILED, tile, [(200, 256, 136), (129, 128, 260), (300, 768, 200), (16, 384, 64)], seed=11)
    _gemm_batch(N, M, bits, TILED, tile, [(520, 256, 256), (520, 256, 256), (520, 256, 192)], seed=12, shared_x=True)


@pytest.mark.parametrize("layout,N,M,bits,shapes", [
    (ROWS, 2, 4, 8, [(70, 256, 136), (33, 128, 64)]),              # row layout: one launch per item
    (ROWS, 3, 4, 8, [(33, 40, 18), (7, 12, 5)]),                   # generic kernel
    (TILED, 2, 4, 8, [(129, 128, 130), (64, 256, 64)]),            # O % 4 != 0 in one item: the batch goes item by item
    (TILED, 2, 8, 4, [(77, 384, 96)]),                             # a batch of one
])
def test_gemm_batch_falls_back_to_one_launch_per_item(layout, N, M, bits, shapes):
    _gemm_batch(N, M, bits, layout, 0, shapes, seed=13)


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 8, 4), (4, 4, 8), (7, 8, 4)])
def test_gemm_tiled_kernels_smallest_shapes(N, M, bits):
    """The smallest problems the matrix-core kernels of the tiled layout accept: one token, four output columns,
    one 128-column slice; one token against a long reduction; a single column tile of 4 with many tokens."""
    _gemm_small(N, M, bits, 0, TILED, shapes=[(1, 128, 4), (1, 4096, 8), (300, 128, 4), (2, 256, 20), (17, 128, 100)], seed=9)


def test_gemm_batch_replayed_from_a_graph():
    """Query / key / value as one nm_gemm_batch launch captured in a HIP graph: the item table lives in
    host memory that is read during the call only, so replays on new activations (same buffers) must
    give the new results."""
    say("gemm batch in a graph")
    N, M, bits, T, K = 2, 4, 8, 520, 768
    rng = np.random.default_rng(77)
    Os = [256, 256, 192]
    Ws = [(rng.standard_normal((O, K)) * 0.02).astype(np.float32) for O in Os]
    refs = [oracle.compress(W, N, M, bits) for W in Ws]
    packed = [gpu_compress(W, N, M, bits, layout=TILED) for W in Ws]
    biases = [(rng.standard_normal(O) * 0.02).astype(np.float32) for O in Os]
    X = torch.zeros((T, K), dtype=torch.int8, device=DEV)
    sx_dev = torch.ones(1, dtype=torch.float32, device=DEV)
    accs = [torch.zeros((T, O), dtype=torch.int32, device=DEV) for O in Os]
    outs = [torch.zeros((T, O), dtype=torch.float32, device=DEV) for O in Os]
    bdev = [torch.from_numpy(b).to(DEV) for b in biases]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    def enqueue(st):
        calls = [dict(X=X, act_scale=0.0, act_scale_dev=sx_dev, vals=p[0], meta=p[1], scales=p[2], O=O, bias=b, acc=a, out=o)
                 for p, O, b, a, o in zip(packed, Os, bdev, accs, outs)]
        nm.nm_gemm_batch(calls, N, M, bits, out_dtype=NM_OUT_F32, layout=TILED, stream=st)

    with torch.cuda.stream(side):
        enqueue(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        Xq, sx = synth.quantize_activations((rng.standard_normal((T, K)) * (1.0 + rep)).astype(np.float32))
        X.copy_(torch.from_numpy(Xq))
        sx_dev.fill_(float(sx))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, O in enumerate(Os):
            acc_ref = oracle.gemm_sparse(Xq, refs[i][0], refs[i][1], O, N, M, bits)
            check_outputs(acc_ref, sx, refs[i][2], biases[i], accs[i].cpu().numpy(), outs[i].cpu().numpy(), None, what="replay %d item %d" % (rep, i))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("N,M,bits", ALL_SCHEMES)
def test_gemm_generic_path_odd_shapes(N, M, bits, layout):
    say("gemm generic", N, M, bits, "layout", layout)
    shapes = [(1, M, 1), (7, 3 * M, 5), (33, 40, 18), (3, 136, 129)] if layout == ROWS else [(1, 128, 1), (33, 128, 18), (3, 256, 129)]
    for T, K, O in shapes:
        if K % M:
            continue
        W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 2)
        packed = gpu_compress(W, N, M, bits, layout=layout)
        assert_packed_equal(packed, oracle_packed(W, N, M, bits, layout), "compress")
        res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32", "bf16"), layout=layout)
        check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], res["bf16"], what="T%d K%d O%d" % (T, K, O))


def test_gemm_large_output_written_through_with_padded_rows():
    """A bf16 output large enough (>= 14 MB) to take the written-through stores of the wide tile, with
    padded output rows (the padding must stay untouched) and a ragged last column tile."""
    say("gemm large output, padded rows")
    T, K, O = 4096, 256, 2240          # 12 column tiles of 192, the last one 128 wide; 18.4 MB of bf16
    W, Xq, sx, bias, ref, acc_ref = small_case(2, 4, 8, T, K, O, 5)
    packed = gpu_compress(W, 2, 4, 8, layout=TILED)
    b16 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("bf16",), ldo=O + 64, layout=TILED)["bf16"]
    assert np.all(b16[:, O:] == 0xC0E0)            # -7.0 in bf16: the padding is as the caller left it
    check_outputs(acc_ref, sx, ref[2], bias, None, None, b16[:, :O], what="bf16 through, padded")
    f32 = run_gemm(Xq, sx, packed, O, 2, 4, 8, bias, want=("f32only",), ldo=O + 64, layout=TILED)["f32only"]
    assert np.all(f32[:, O:] == -7.0)
    check_outputs(acc_ref, sx, ref[2], bias, None, f32[:, :O], None, what="f32 through, padded")


@pytest.mark.parametrize("layout", LAYOUTS)
def test_gemm_padded_output_rows_and_no_bias(layout):
    W, Xq, sx, _, ref, acc_ref = small_case(2, 4, 8, 150, 256, 128, 3, with_bias=False)
    packed = gpu_compress(W, 2, 4, 8, layout=layout)
    res = run_gemm(Xq, sx, packed, 128, 2, 4, 8, None, want=("acc", "f32", "bf16"), ldo=160, layout=layout)
    assert np.all(res["acc"][:, 128:] == -7) and np.all(res["f32"][:, 128:] == -7.0)   # padding untouched
    check_outputs(acc_ref, sx, ref[2], None, res["acc"][:, :128], res["f32"][:, :128], res["bf16"][:, :128])


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (4, 4, 8)])
def test_gemm_extreme_codes_do_not_overflow(N, M, bits, layout):
    K, O, T = 4096, 16, 16
    W = np.ones((O, K), np.float32)
    Xq = np.full((T, K), -127, np.int8)
    packed = gpu_compress(W, N, M, bits, layout=layout)
    res = run_gemm(Xq, 1.0, packed, O, N, M, bits, None, want=("acc",), layout=layout)
    assert np.all(res["acc"] == -127 * 127 * (K * N // M))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_sparse_product_equals_dense_product_on_gpu(layout):
    W, Xq, sx, _, ref, acc_ref = small_case(2, 4, 8, 256, 512, 256, 4, with_bias=False)
    packed = gpu_compress(W, 2, 4, 8, layout=layout)
    Wq = nm.nm_decompress_i8(packed[0], packed[1], 256, 512, 2, 4, 8, layout=layout)
    dense = (torch.from_numpy(Xq).to(DEV).float() @ Wq.float().T).round().to(torch.int32)   # exact: |sum| < 2^24
    res = run_gemm(Xq, sx, packed, 256, 2, 4, 8, None, want=("acc",), layout=layout)
    assert np.array_equal(res["acc"], dense.cpu().numpy())


# ---- the five workloads -----------------------------------------------------------------------

@pytest.mark.parametrize("layout", LAYOUTS)
def test_config1_full(layout):
    g, W, Xq, sx = synth.config1_tensors()
    ref = oracle.compress(W, g.N, g.M, g.bits)
    packed = gpu_compress(W, g.N, g.M, g.bits, layout=layout)
    assert_packed_equal(packed, oracle_packed(W, g.N, g.M, g.bits, layout), "config 1")
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], g.O, g.N, g.M, g.bits)
    res = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc", "f32", "bf16", "f32only"), layout=layout)
    check_outputs(acc_ref, sx, ref[2], None, res["acc"], res["f32"], res["bf16"], what="config 1")
    check_outputs(acc_ref, sx, ref[2], None, None, res["f32only"], None, what="config 1, f32 alone")


def stratified_tokens(T, per_block=2, block=64, seed=0):
    """Token rows to compare at full size: `per_block` random rows of every block of 64 tokens,
    so that every token tile of every tile shape (64 to 256 rows) has compared rows, plus the
    rows next to the tile edges at both ends."""
    rng = np.random.default_rng(seed)
    rows = [np.array([0, 1, 15, 16, 63, 64, 127, 128, 191, 192, 255, 256, T - 257, T - 256, T - 129, T - 128, T - 17, T - 2, T - 1])]
    for b0 in range(0, T, block):
        rows.append(b0 + rng.integers(0, min(block, T - b0), size=per_block))
    rows = np.unique(np.concatenate(rows))
    return rows[(rows >= 0) & (rows < T)]


def full_size_case(g, layout, rows=None):
    """Whole compress compared byte for byte; GEMM compared on the given token rows (all of them
    when `rows` is None), which the oracle computes one by one, in the launch configuration the
    library picks for the full size: accumulators + fp32 in one call, bf16 alone, fp32 alone."""
    say("full size", g, "layout", layout, "rows", "all" if rows is None else len(rows))
    W = synth.weights(g)
    Xq, sx = synth.activations(g)
    bias = synth.bias(g)
    ref = oracle.compress(W, g.N, g.M, g.bits)
    packed = gpu_compress(W, g.N, g.M, g.bits, layout=layout)
    assert_packed_equal(packed, oracle_packed(W, g.N, g.M, g.bits, layout), g.name)
    if rows is None:
        rows = np.arange(g.T)
    acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
    res = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, bias, want=("acc", "f32", "bf16", "f32only"), layout=layout)
    check_outputs(acc_ref, sx, ref[2], bias, res["acc"][rows], res["f32"][rows], res["bf16"][rows], what=str(g))
    check_outputs(acc_ref, sx, ref[2], bias, None, res["f32only"][rows], None, what=str(g) + " f32 alone")
    # every output element was written (the buffers were pre-filled with a sentinel)
    for k in ("f32", "f32only"):
        assert np.count_nonzero(res[k] == -7.0) < 4
    assert np.count_nonzero(res["bf16"] == 0xC0E0) < max(64, 4e-6 * res["bf16"].size)     # -7.0 is a value bf16 outputs do take now and then


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(4))
def test_config2_bert_base_2of4_int8_every_token(i, layout):
    full_size_case(synth.config2()[i], layout)


@pytest.mark.parametrize("i", range(4))
def test_config3_bert_large_2of4_int8(i):
    g = synth.config3()[i]
    full_size_case(g, TILED, stratified_tokens(g.T, seed=i))


@pytest.mark.parametrize("i", range(8))
def test_config4_int4_1of4_and_2of8(i):
    g = synth.config4()[i]
    full_size_case(g, TILED, stratified_tokens(g.T, seed=10 + i))


def test_config4_row_layout():
    for i in (2, 7):
        g = synth.config4()[i]
        full_size_case(g, ROWS, stratified_tokens(g.T, seed=20 + i))


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
        packed = nm.nm_compress(torch.from_numpy(W).to(DEV), g.N, g.M, g.bits, layout=TILED)
        Xq, sx = acts[g.K]
        X = torch.from_numpy(Xq).to(DEV)
        acc = torch.empty((g.T, g.O), dtype=torch.int32, device=DEV)
        out = torch.empty((g.T, g.O), dtype=torch.bfloat16, device=DEV)
        jobs.append((g, ref, packed, X, sx, acc, out))
    torch.cuda.synchronize()
    for g, ref, packed, X, sx, acc, out in jobs:          # all 48 launches back to back on one stream
        nm.nm_gemm(X, float(sx), *packed, g.O, g.N, g.M, g.bits, acc=acc, out=out, out_dtype=NM_OUT_BF16, stream=stream, layout=TILED)
    torch.cuda.synchronize()
    for g, ref, packed, X, sx, acc, out in jobs:
        vt, mt = oracle.to_tiled(ref[0], ref[1], g.K, g.N, g.M, g.bits)
        assert_packed_equal(packed, (vt, mt, ref[2]), str(g))
        rows = stratified_tokens(g.T, seed=g.seed[1] * 4 + g.seed[2])
        Xq = acts[g.K][0]
        acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
        check_outputs(acc_ref, sx, ref[2], None, acc.cpu().numpy()[rows], None,
                      out.view(torch.int16).cpu().numpy().view(np.uint16)[rows], what=str(g))


def test_results_do_not_depend_on_repetition():
    g = synth.config2()[3]
    W, (Xq, sx) = synth.weights(g), synth.activations(g)
    packed = gpu_compress(W, g.N, g.M, g.bits, layout=TILED)
    a = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",), layout=TILED)["acc"]
    b = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",), layout=TILED)["acc"]
    assert np.array_equal(a, b)


@pytest.mark.parametrize("N,M,bits", [(4, 4, 8), (4, 4, 4), (3, 4, 8), (4, 8, 8), (4, 8, 4)])
def test_dense_and_three_of_four_at_bert_base_size(N, M, bits):
    """The dense Q8 / Q4 components of the heterogeneous configurations (Sec. 5.4) and the patterns
    with more than two kept entries per group, on the BERT-base FFN shapes at 4096 tokens, in the
    launch configuration the library picks."""
    import dataclasses
    for g in synth.config2()[2:]:
        g = dataclasses.replace(g, N=N, M=M, bits=bits, seed=(6, N * 10 + M, bits))
        full_size_case(g, TILED, stratified_tokens(g.T, seed=N + bits))


@pytest.mark.parametrize("T", [128, 384, 8192, 16384, 24576, 49152])
def test_inference_table_token_counts_bert_large(T):
    """Token counts of the paper's inference table (Sec. 5.3: batch {1, 32, 64, 128} x sequence {128, 384}) that the
    workloads above do not cover, on the BERT-large layer set: the tile choice differs with the token count."""
    import dataclasses
    for g in synth.config3():
        if T > 16384 and g.name in ("qkv", "attn_out"):
            continue                               # the two largest counts: the FFN pair (both reduction widths, both tile families)
        g = dataclasses.replace(g, T=T)
        full_size_case(g, TILED, stratified_tokens(g.T, per_block=1 if T > 4096 else 2, block=64 if T <= 16384 else 128, seed=T % 97))


# ---- requantised output (nm_gemm_q8) -------------------------------------------------------------
def run_gemm_q8(Xq, sx, packed, O, N, M, bits, bias, out_scale, ldo=None, start_max=0.0, layout=ROWS, device_scales=False):
    vals, meta, scales = packed
    X = torch.from_numpy(Xq).to(DEV)
    T = Xq.shape[0]
    ldo = ldo or O
    b = None if bias is None else torch.from_numpy(bias).to(DEV)
    out = torch.full((T, ldo), -77, dtype=torch.int8, device=DEV)
    amax = torch.full((1,), start_max, dtype=torch.float32, device=DEV)
    if device_scales:                          # the host values are then decoys
        sa = torch.tensor([float(sx)], dtype=torch.float32, device=DEV)
        so = torch.tensor([float(out_scale)], dtype=torch.float32, device=DEV)
        nm.nm_gemm_q8(X, 123.0, vals, meta, scales, O, N, M, bits, 456.0, out, bias=b, absmax=amax, ldo=ldo, layout=layout,
                      act_scale_dev=sa, out_scale_dev=so)
    else:
        nm.nm_gemm_q8(X, float(sx), vals, meta, scales, O, N, M, bits, float(out_scale), out, bias=b, absmax=amax, ldo=ldo, layout=layout)
    torch.cuda.synchronize()
    return out.cpu().numpy(), float(amax.item())


def check_q8(acc_ref, sx, scales_ref, bias, out_scale, q_gpu, amax_gpu, what=""):
    """The oracle divides every dequantised output by the scale (Eq. 4, then Eq. 5); the kernel folds
    the division into per-column constants, which moves the quotient by less than
    1e-6 * (|acc| s_act s_w + |bias|) / s_out (six fp32 roundings of 2^-24 each).  So: codes equal,
    except where the oracle's quotient lies within that distance of a half-way point k + 1/2 -
    there one step apart at most - and such places are rare; max |y| within the same bound."""
    q_ref, amax_ref = oracle.requant(acc_ref, float(sx), scales_ref, float(out_scale), bias)
    f32, _ = oracle.dequant(acc_ref, float(sx), scales_ref, bias)
    mag = np.abs(acc_ref).astype(np.float64) * float(sx) * scales_ref[None, :].astype(np.float64)
    if bias is not None:
        mag = mag + np.abs(bias)[None, :].astype(np.float64)
    band = 1e-6 * mag / float(out_scale)
    t = f32.astype(np.float64) / float(out_scale)
    near_half = np.abs(t - np.floor(t) - 0.5) <= band
    differ = q_gpu != q_ref
    assert not np.any(differ & ~near_half), "%s: %d codes differ away from any half-way point" % (what, np.count_nonzero(differ & ~near_half))
    assert np.all(np.abs(q_gpu.astype(np.int32) - q_ref.astype(np.int32)) <= 1), what
    assert np.count_nonzero(differ) <= 2e-3 * differ.size + 2, "%s: %d of %d codes differ" % (what, np.count_nonzero(differ), differ.size)
    assert abs(amax_gpu - amax_ref) <= 1e-6 * mag.max() + 1e-37, "%s: max |y| %r against %r" % (what, amax_gpu, amax_ref)


def q8_scale(acc_ref, sx, scales_ref, bias):
    """An output scale that uses the code range: max |y| / 127, as a caller would choose it."""
    f32, _ = oracle.dequant(acc_ref, float(sx), scales_ref, bias)
    return np.float32(np.abs(f32).max() / 127.0)


@pytest.mark.parametrize("tile,layout", [(0, ROWS), (2, ROWS), (0, TILED), (113, TILED), (116, TILED), (122, TILED), (133, TILED), (136, TILED)])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 4, 4), (2, 8, 4), (4, 4, 8)])
def test_gemm_q8_fast_paths(N, M, bits, tile, layout):
    """Every kernel family, whole and ragged tiles, rows of 16-byte, 8-byte and 4-byte granularity, with and
    without bias, scales from the host and from device memory."""
    say("gemm q8", N, M, bits, "tile", tile, "layout", layout)
    with forced_tile(tile):
        for T, K, O, with_bias, pad in [(300, 256, 392, True, 0), (129, 512, 260, False, 0), (512, 768, 768, True, 8), (16, 384, 64, True, 4), (300, 256, 384, True, 16)]:
            W, Xq, sx, bias, ref, acc_ref = small_case(N, M, bits, T, K, O, 21, with_bias=with_bias)
            packed = gpu_compress(W, N, M, bits, layout=layout)
            so = q8_scale(acc_ref, sx, ref[2], bias)
            q, amax = run_gemm_q8(Xq, sx, packed, O, N, M, bits, bias, so, ldo=O + pad, layout=layout, device_scales=(T == 300))
            assert np.all(q[:, O:] == -77)                 # padding untouched
            check_q8(acc_ref, sx, ref[2], bias, so, q[:, :O], amax, what="T%d K%d O%d" % (T, K, O))


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
    packed = gpu_compress(W, 2, 4, 8, layout=TILED)
    so = q8_scale(acc_ref, sx, ref[2], bias)
    _, amax_ref = oracle.requant(acc_ref, float(sx), ref[2], float(so), bias)
    _, amax = run_gemm_q8(Xq, sx, packed, 96, 2, 4, 8, bias, so, start_max=amax_ref * 4.0, layout=TILED)
    assert amax == np.float32(amax_ref * 4.0)              # a larger value already there survives
    _, amax = run_gemm_q8(Xq, sx, packed, 96, 2, 4, 8, bias, so, start_max=amax_ref / 4.0, layout=TILED)
    assert abs(amax - amax_ref) <= 1e-5 * amax_ref


def test_gemm_q8_full_size_layer_feeds_the_next_one():
    """BERT-base FFN-up at 4096 tokens in the configuration the benchmark uses, its codes checked in
    full, then used as the activations of FFN-down: the chain never leaves int8."""
    say("gemm q8 full size")
    g_up, g_down = [g for g in synth.config2() if g.name in ("ffn_up", "ffn_down")]
    W = synth.weights(g_up); Xq, sx = synth.activations(g_up); bias = synth.bias(g_up)
    ref = oracle.compress(W, 2, 4, 8)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], g_up.O, 2, 4, 8)
    packed = gpu_compress(W, 2, 4, 8, layout=TILED)
    so = q8_scale(acc_ref, sx, ref[2], bias)
    q, amax = run_gemm_q8(Xq, sx, packed, g_up.O, 2, 4, 8, bias, so, layout=TILED)
    check_q8(acc_ref, sx, ref[2], bias, so, q, amax, what="ffn_up")
    W2 = synth.weights(g_down)
    ref2 = oracle.compress(W2, 2, 4, 8)
    acc2_ref = oracle.gemm_sparse(q, ref2[0], ref2[1], g_down.O, 2, 4, 8)     # on the codes the GPU produced
    packed2 = gpu_compress(W2, 2, 4, 8, layout=TILED)
    res = run_gemm(q, so, packed2, g_down.O, 2, 4, 8, None, want=("acc",), layout=TILED)
    assert np.array_equal(res["acc"], acc2_ref)


def test_int8_chain_with_device_scales_replayed_from_a_graph():
    """FFN-up -> FFN-down captured once in a HIP graph, every scale between the two layers living in device
    memory: FFN-up writes int8 codes with the scale that nm_absmax_to_scale derived from the max |y| of the
    replay before, FFN-down reads that same device scale as its activation scale.  Replayed on changing
    inputs (eager work and synchronisations in between); every replay is checked against the oracle chain
    requant(scale = previous max |y| / 127) -> sparse product -> dequantisation."""
    say("graph replay: int8 chain on device scales")
    N, M, bits = 2, 4, 8
    T, H, F = 320, 256, 1024
    rng = np.random.default_rng(41)
    W1 = (rng.standard_normal((F, H)) * 0.02).astype(np.float32)
    W2 = (rng.standard_normal((H, F)) * 0.02).astype(np.float32)
    b1 = (rng.standard_normal(F) * 0.02).astype(np.float32)
    r1, r2 = oracle.compress(W1, N, M, bits), oracle.compress(W2, N, M, bits)
    p1 = nm.nm_compress(torch.from_numpy(W1).to(DEV), N, M, bits, layout=TILED)
    p2 = nm.nm_compress(torch.from_numpy(W2).to(DEV), N, M, bits, layout=TILED)
    X = torch.zeros((T, H), dtype=torch.int8, device=DEV)
    sx_dev = torch.ones(1, dtype=torch.float32, device=DEV)
    mid = torch.zeros((T, F), dtype=torch.int8, device=DEV)
    y = torch.zeros((T, H), dtype=torch.float32, device=DEV)
    acc2 = torch.zeros((T, H), dtype=torch.int32, device=DEV)
    amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    s_mid = torch.ones(1, dtype=torch.float32, device=DEV)
    b1d = torch.from_numpy(b1).to(DEV)

    def enqueue(st):
        nm.nm_absmax_to_scale(amax, s_mid, reset=True, stream=st)           # scale from the statistic of the step before
        nm.nm_gemm_q8(X, 0.0, *p1, F, N, M, bits, 0.0, mid, bias=b1d, absmax=amax, stream=st, layout=TILED,
                      act_scale_dev=sx_dev, out_scale_dev=s_mid)
        nm.nm_gemm(mid, 0.0, *p2, H, N, M, bits, acc=acc2, out=y, out_dtype=NM_OUT_F32, stream=st, layout=TILED, act_scale_dev=s_mid)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enqueue(side)                                                       # warm-up, leaves a statistic behind
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    prev_amax = float(amax.item())
    for rep in range(4):
        Xq, sx = synth.quantize_activations((rng.standard_normal((T, H)) * (1.0 + rep)).astype(np.float32))
        X.copy_(torch.from_numpy(Xq))
        sx_dev.fill_(float(sx))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        s_ref = np.float32(1.0) if prev_amax == 0.0 else np.float32(prev_amax) / np.float32(127.0)
        assert float(s_mid.item()) == float(s_ref), "replay %d: scale %r against %r" % (rep, float(s_mid.item()), float(s_ref))
        acc1_ref = oracle.gemm_sparse(Xq, r1[0], r1[1], F, N, M, bits)
        q_gpu = mid.cpu().numpy()
        check_q8(acc1_ref, sx, r1[2], b1, s_ref, q_gpu, float(amax.item()), what="replay %d, first layer" % rep)
        acc2_ref = oracle.gemm_sparse(q_gpu, r2[0], r2[1], H, N, M, bits)
        check_outputs(acc2_ref, s_ref, r2[2], None, acc2.cpu().numpy(), y.cpu().numpy(), None, what="replay %d, second layer" % rep)
        prev_amax = float(amax.item())
        assert prev_amax > 0


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
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("rps", [2, 32, 100])
@pytest.mark.parametrize("N,M,bits", FAST_SCHEMES + [(3, 4, 8), (4, 8, 4), (4, 4, 4)])
def test_compress_grouped_matches_oracle_and_feeds_the_gemm(N, M, bits, rps, layout):
    say("compress grouped", N, M, bits, "rows per scale", rps, "layout", layout)
    rng = np.random.default_rng([N, M, bits, rps, 3])
    for rows, cols, ldw in [(70, 256, None), (257, 1408, None), (768, 768, 776), (5, 8 * M, None), (33, 40, None)]:
        if cols % M or (layout == TILED and cols % 128):
            continue
        W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
        W[rng.integers(0, rows)] = 0.0
        ref = oracle_packed(W, N, M, bits, layout, rows_per_scale=rps)
        Wt = torch.from_numpy(W).to(DEV)
        if ldw is not None:
            buf = torch.zeros((rows, ldw), dtype=torch.float32, device=DEV)
            buf[:, :cols] = Wt
            Wt = buf[:, :cols]
        packed = nm.nm_compress_grouped(Wt, N, M, bits, rps, layout=layout)
        torch.cuda.synchronize()
        assert_packed_equal(packed, ref, "grouped %dx%d" % (rows, cols))
    # the packed result is an ordinary operand of nm_gemm
    T, K, O = 200, 256, 136
    W, Xq, sx, bias, _, _ = small_case(N, M, bits, T, K, O, 4)
    ref = oracle.compress_grouped(W, N, M, bits, rps)
    acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
    packed = nm.nm_compress_grouped(torch.from_numpy(W).to(DEV), N, M, bits, rps, layout=layout)
    res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32"), layout=layout)
    check_outputs(acc_ref, sx, ref[2], bias, res["acc"], res["f32"], None, what="gemm on grouped scales")


# ---- the distance-minimising scale rule (nm_scale_search) and compress with given scales -----------
@pytest.mark.parametrize("rps", [1, 32, 70])
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 4), (2, 8, 4), (4, 4, 4), (3, 4, 8), (4, 8, 8)])
def test_scale_search_matches_oracle_and_feeds_compress(N, M, bits, rps):
    """Scales equal to the oracle's, bit for bit - except where the oracle's own errors of the two
    candidates agree to 1e-12 relative (the sums run in different orders on the two sides; either choice
    is then a correct minimiser); then nm_compress_scaled with those scales against the oracle, byte for
    byte in both layouts, and the result through nm_gemm."""
    say("scale search", N, M, bits, "rows per scale", rps)
    rng = np.random.default_rng([N, M, bits, rps, 12])
    C = 32
    for rows, cols, ldw in [(70, 256, None), (257, 768, 776), (5, 8 * M, None), (768, 768, None)]:
        W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
        W[rng.integers(0, rows)] = 0.0
        W[::7] *= np.linspace(0.05, 4.0, cols).astype(np.float32)           # heavy-tailed rows: a smaller scale pays
        s_ref, err = oracle.dist_scales(W, N, M, bits, rps, C)
        Wt = torch.from_numpy(W).to(DEV)
        if ldw is not None:
            buf = torch.zeros((rows, ldw), dtype=torch.float32, device=DEV)
            buf[:, :cols] = Wt
            Wt = buf[:, :cols]
        s_dev = nm.nm_scale_search(Wt, N, M, bits, rps, C)
        torch.cuda.synchronize()
        s_gpu = s_dev.cpu().numpy()
        qmax = (1 << (bits - 1)) - 1
        for gi, r0 in enumerate(range(0, rows, rps)):
            blk = slice(r0, min(r0 + rps, rows))
            assert np.all(s_gpu[blk] == s_gpu[r0])
            if s_gpu[r0] == s_ref[r0]:
                continue
            amax = np.abs(W[blk]).max()
            smax = np.float32(amax) / np.float32(qmax)
            cands = [np.float32(np.float32(smax * np.float32(c)) / np.float32(C)) for c in range(C // 2, C + 1)]
            assert s_gpu[r0] in cands, "group %d: %r is no candidate" % (gi, s_gpu[r0])
            e_gpu, e_ref = err[gi][cands.index(s_gpu[r0])], err[gi].min()
            assert e_gpu <= e_ref * (1 + 1e-12), "group %d: chose error %r, least is %r" % (gi, e_gpu, e_ref)
        if bits == 4 and rows >= 70:
            assert np.any(s_gpu < np.abs(W).max(axis=1) / np.float32(qmax) * 0.99)     # the search does move scales
        if cols % 128 == 0:
            for layout in LAYOUTS:
                packed = nm.nm_compress_scaled(Wt, N, M, bits, s_dev, layout=layout)
                torch.cuda.synchronize()
                v, m = oracle.compress_scaled(W, N, M, bits, s_gpu)
                if layout == TILED:
                    v, m = oracle.to_tiled(v, m, cols, N, M, bits)
                assert_packed_equal(packed, (v, m, s_gpu), "scaled %dx%d layout %d" % (rows, cols, layout))
    T, K, O = 200, 256, 136
    W, Xq, sx, bias, _, _ = small_case(N, M, bits, T, K, O, 14)
    Wt = torch.from_numpy(W).to(DEV)
    s_dev = nm.nm_scale_search(Wt, N, M, bits, rps, C)
    packed = nm.nm_compress_scaled(Wt, N, M, bits, s_dev, layout=TILED)
    torch.cuda.synchronize()
    v, m = oracle.compress_scaled(W, N, M, bits, s_dev.cpu().numpy())
    acc_ref = oracle.gemm_sparse(Xq, v, m, O, N, M, bits)
    res = run_gemm(Xq, sx, packed, O, N, M, bits, bias, want=("acc", "f32"), layout=TILED)
    check_outputs(acc_ref, sx, s_dev.cpu().numpy(), bias, res["acc"], res["f32"], None, what="gemm on searched scales")


# ---- several matrices in one call (nm_compress_batch): byte for byte what nm_compress gives -----
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 4, 4), (2, 8, 4), (4, 8, 8), (3, 4, 8), (4, 4, 8), (8, 8, 4)])
def test_compress_batch_matches_oracle_item_by_item(N, M, bits, layout):
    """Matrices of different heights and widths in one call: one, two and four wavefronts per row
    (widths up to 3072), heights that are not multiples of the rows per workgroup (nor of the 16
    rows of a block of the tiled layout), a padded leading dimension, a matrix whose packed rows
    are not whole dwords (row layout only; goes out on its own), more matrices than one launch
    takes (17 of them follow), and 3:4, which no wavefront kernel covers."""
    say("compress batch", N, M, bits, "layout", layout)
    rng = np.random.default_rng([N, M, bits, 77])
    shapes = [(37, 768, 768), (5, 3072, 3072), (130, 1536, 1600), (9, 5 * M, 5 * M), (64, 256, 256)] + [(3 + i, 128, 128) for i in range(17)]
    if layout == TILED:
        shapes = [sh for sh in shapes if sh[1] % 128 == 0]
    Ws, dev = [], []
    for rows, cols, ldw in shapes:
        W = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
        W[rows // 2, :] = 0.0                                  # an all-zero row: scale 1
        buf = torch.zeros((rows, ldw), dtype=torch.float32, device=DEV)
        buf[:, :cols] = torch.from_numpy(W).to(DEV)
        Ws.append(W)
        dev.append(buf[:, :cols])
    outs = []
    for W in Ws:                                               # pre-filled: bytes left out would show
        vb, mb, _ = nm.nm_packed_sizes(W.shape[0], W.shape[1], N, M, bits, layout)
        shape = (lambda n: (W.shape[0], n // W.shape[0])) if layout == ROWS else (lambda n: (n,))
        outs.append((torch.full(shape(vb), 0x5A, dtype=torch.uint8, device=DEV), torch.full(shape(mb), 0x5A, dtype=torch.uint8, device=DEV),
                     torch.empty(W.shape[0], dtype=torch.float32, device=DEV)))
    outs = nm.nm_compress_batch(dev, N, M, bits, outs=outs, layout=layout)
    torch.cuda.synchronize()
    for W, packed, shape in zip(Ws, outs, shapes):
        assert_packed_equal(packed, oracle_packed(W, N, M, bits, layout), "batch item %s" % (shape,))


def test_compress_batch_full_size_layer_set_feeds_the_gemm():
    gs = synth.config2()
    Ws = [synth.weights(g) for g in gs]
    outs = nm.nm_compress_batch([torch.from_numpy(W).to(DEV) for W in Ws], 2, 4, 8, layout=TILED)
    torch.cuda.synchronize()
    for g, W, packed in zip(gs, Ws, outs):
        assert_packed_equal(packed, oracle_packed(W, g.N, g.M, g.bits, TILED), "batch " + g.name)
    g, W, packed = gs[1], Ws[1], outs[1]
    Xq, sx = synth.activations(g)
    rows = stratified_tokens(g.T, per_block=1, seed=5)
    ref = oracle.compress(W, g.N, g.M, g.bits)
    acc_ref = oracle.gemm_sparse(Xq[rows], ref[0], ref[1], g.O, g.N, g.M, g.bits)
    acc = run_gemm(Xq, sx, packed, g.O, g.N, g.M, g.bits, None, want=("acc",), layout=TILED)["acc"]
    assert np.array_equal(acc[rows], acc_ref)


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (2, 4, 4), (1, 4, 8), (2, 8, 4), (4, 4, 8)])
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
    for layout in LAYOUTS:
        packed = gpu_compress(W, N, M, bits, layout=layout)
        assert_packed_equal(packed, oracle_packed(W, N, M, bits, layout), "half-way quotients")


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
    outs = nm.nm_compress_batch(Wd, N, M, bits, layout=TILED)             # allocates the packed buffers (and warms up)
    T, K, O = 200, 256, 96
    Xq, sx = synth.quantize_activations(rng.standard_normal((T, K)).astype(np.float32))
    X = torch.from_numpy(Xq).to(DEV)
    acc = torch.empty((T, O), dtype=torch.int32, device=DEV)
    y = torch.empty((T, O), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        nm.nm_gemm(X, float(sx), *outs[0], O, N, M, bits, acc=acc, out=y, out_dtype=NM_OUT_F32, stream=side, layout=TILED)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            nm.nm_compress_batch(Wd, N, M, bits, outs=outs, stream=side, layout=TILED)
            nm.nm_gemm(X, float(sx), *outs[0], O, N, M, bits, acc=acc, out=y, out_dtype=NM_OUT_F32, stream=side, layout=TILED)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for W, d in zip(Ws, Wd):                            # new weights in the same buffers
            W[...] = (rng.standard_normal(W.shape) * 0.02 * (rep + 1)).astype(np.float32)
            d.copy_(torch.from_numpy(W))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for W, packed in zip(Ws, outs):
            assert_packed_equal(packed, oracle_packed(W, N, M, bits, TILED), "replay %d" % rep)
        ref = oracle.compress(Ws[0], N, M, bits)
        acc_ref = oracle.gemm_sparse(Xq, ref[0], ref[1], O, N, M, bits)
        check_outputs(acc_ref, sx, ref[2], None, acc.cpu().numpy(), y.cpu().numpy(), None, what="replay %d" % rep)


# ---- floating-point activations -> 8-bit codes (nm_absmax_f32, nm_quantize_act) ----

def _act_buffers(X, ldx, ldq, x_off=0, q_off=0):
    """Device copies of X with row stride ldx starting x_off floats into a 16-byte aligned allocation, and an
    int8 output of row stride ldq starting q_off bytes in, pre-filled with 77 so that stray writes show."""
    T, K = X.shape
    xbuf = torch.zeros(x_off + T * ldx, dtype=torch.float32, device=DEV)
    Xd = xbuf[x_off:x_off + T * ldx].view(T, ldx)[:, :K]
    Xd.copy_(torch.from_numpy(X))
    qbuf = torch.full((q_off + T * ldq,), 77, dtype=torch.int8, device=DEV)
    Qd = qbuf[q_off:q_off + T * ldq].view(T, ldq)[:, :K]
    return Xd, Qd, qbuf


ACT_SHAPES = [
    # tokens, K, ldx, ldq, x_off, q_off
    (384, 768, 768, 768, 0, 0),          # a layer's input, one long row of 16-byte pieces
    (7, 36, 36, 36, 0, 0),               # far less than one workgroup
    (4, 33, 33, 33, 0, 0),               # rows are not whole pieces, the tensor is
    (5, 33, 33, 33, 0, 0),               # nothing is: one element per lane
    (130, 4100, 4104, 4112, 0, 0),       # padded rows of whole pieces, ragged against the block width
    (130, 4100, 4104, 4112, 4, 8),       # ... starting a piece further in
    (61, 250, 253, 251, 1, 3),           # odd strides and offsets
    (70000, 8, 12, 8, 0, 0),             # more rows than the grid has: the row loop
    (1, 1, 1, 1, 0, 0),
]


@pytest.mark.parametrize("T,K,ldx,ldq,x_off,q_off", ACT_SHAPES)
def test_quantize_act_matches_oracle(T, K, ldx, ldq, x_off, q_off):
    """max |x| -> scale -> codes, every scale on the device, against the oracle's quantiser: scale and codes bit-exact,
    padding of the output untouched."""
    say("quantize_act", T, K, ldx, ldq, x_off, q_off)
    rng = np.random.default_rng(T * 131 + K)
    X = (rng.standard_normal((T, K)) * rng.choice([0.01, 1.0, 40.0])).astype(np.float32)
    X[rng.integers(T), rng.integers(K)] *= 3.0                               # one clear maximum somewhere
    Q_ref, s_ref = oracle.quantize_act(X)
    Xd, Qd, qbuf = _act_buffers(X, ldx, ldq, x_off, q_off)
    amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    s_dev = torch.zeros(1, dtype=torch.float32, device=DEV)
    nm.nm_absmax_f32(Xd, amax)
    nm.nm_absmax_to_scale(amax, s_dev)
    nm.nm_quantize_act(Xd, out=Qd, scale_dev=s_dev)
    torch.cuda.synchronize()
    assert float(amax.item()) == float(np.abs(X).max())
    assert np.float32(s_dev.item()) == s_ref
    assert np.array_equal(Qd.cpu().numpy(), Q_ref)
    full = qbuf.cpu().numpy()
    assert np.all(full[:q_off] == 77)
    pad = full[q_off:].reshape(T, ldq)[:, K:]
    assert np.all(pad == 77)
    # the host scale takes the same decisions as the device one
    Q2 = nm.nm_quantize_act(Xd, scale=float(s_ref))
    assert np.array_equal(Q2.cpu().numpy(), Q_ref)


@pytest.mark.parametrize("scale", [0.5, 2.0 ** -50, 2.0 ** -61, 1e-30, 3.0e-39, 1e30, 2.0 ** 60, 2.0 ** 61, 0.1, 1.0 / 3.0])
@pytest.mark.parametrize("aligned", [True, False])
def test_quantize_act_with_a_caller_scale(scale, aligned):
    """A caller's scale (both division routes of the kernel and the scales between them): half-way quotients, values
    far outside the representable range and tiny ones, against the oracle."""
    say("quantize_act caller scale", scale, aligned)
    s = np.float32(scale)
    rng = np.random.default_rng(9)
    K = 64 if aligned else 63
    steps = np.concatenate([np.arange(-130, 131) + 0.5, np.arange(-130, 131), rng.uniform(-140, 140, 3 * K)]).astype(np.float32)
    with np.errstate(over="ignore", under="ignore"):
        body = (steps * s).astype(np.float32)                                   # exact where s is a power of two
        extremes = np.array([3.0e38, -3.0e38, 1e30, -1e30, 1e-30, -1e-30, 1e-44, 0.0, -0.0, 127.49, -127.51], np.float32)
        flat = np.concatenate([body[np.isfinite(body)], extremes, (extremes * s).astype(np.float32)])
    flat = flat[np.isfinite(flat)]
    flat = np.resize(flat, (len(flat) + K - 1) // K * K)
    X = flat.reshape(-1, K)
    Q_ref, s_used = oracle.quantize_act(X, scale=s)
    assert s_used == s
    Xd, Qd, _ = _act_buffers(X, K, K, 0, 0)
    nm.nm_quantize_act(Xd, scale=float(s), out=Qd)
    torch.cuda.synchronize()
    got = Qd.cpu().numpy()
    bad = np.argwhere(got != Q_ref)
    assert bad.size == 0, "first differences (t, k, x, got, want): %r" % [
        (int(t), int(k), float(X[t, k]), int(got[t, k]), int(Q_ref[t, k])) for t, k in bad[:5]]


def test_absmax_f32_degenerate_and_running_maximum():
    say("absmax_f32 zero tensor / running maximum")
    X = np.zeros((9, 40), np.float32)
    Xd, Qd, _ = _act_buffers(X, 40, 40)
    amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    s_dev = torch.zeros(1, dtype=torch.float32, device=DEV)
    nm.nm_absmax_f32(Xd, amax)
    nm.nm_absmax_to_scale(amax, s_dev)
    nm.nm_quantize_act(Xd, out=Qd, scale_dev=s_dev)
    torch.cuda.synchronize()
    Q_ref, s_ref = oracle.quantize_act(X)
    assert float(amax.item()) == 0.0 and np.float32(s_dev.item()) == s_ref == np.float32(1.0)
    assert np.array_equal(Qd.cpu().numpy(), Q_ref)
    # a statistic shared by two tensors, and one that is already larger than both
    rng = np.random.default_rng(3)
    A = rng.standard_normal((33, 128)).astype(np.float32)
    B = (rng.standard_normal((17, 57)) * 2).astype(np.float32)
    amax.zero_()
    nm.nm_absmax_f32(torch.from_numpy(A).to(DEV), amax)
    nm.nm_absmax_f32(torch.from_numpy(B).to(DEV), amax)
    torch.cuda.synchronize()
    assert float(amax.item()) == float(max(np.abs(A).max(), np.abs(B).max()))
    amax.fill_(1e6)
    nm.nm_absmax_f32(torch.from_numpy(A).to(DEV), amax)
    torch.cuda.synchronize()
    assert float(amax.item()) == float(np.float32(1e6))


def test_quantize_act_feeds_the_sparse_gemm():
    """fp32 activations -> codes and scale on the device -> nm_gemm reading that device scale, against the oracle's
    quantiser, sparse product and dequantisation."""
    say("quantize_act -> nm_gemm")
    N, M, bits = 2, 4, 8
    T, K, O = 200, 256, 320
    rng = np.random.default_rng(77)
    X = rng.standard_normal((T, K)).astype(np.float32)
    W = (rng.standard_normal((O, K)) * 0.02).astype(np.float32)
    ref = oracle.compress(W, N, M, bits)
    Q_ref, s_ref = oracle.quantize_act(X)
    acc_ref = oracle.gemm_sparse(Q_ref, ref[0], ref[1], O, N, M, bits)
    y_ref, _ = oracle.dequant(acc_ref, s_ref, ref[2], None)
    packed = nm.nm_compress(torch.from_numpy(W).to(DEV), N, M, bits, layout=TILED)
    Xd = torch.from_numpy(X).to(DEV)
    amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    s_dev = torch.zeros(1, dtype=torch.float32, device=DEV)
    nm.nm_absmax_f32(Xd, amax)
    nm.nm_absmax_to_scale(amax, s_dev)
    Xq = nm.nm_quantize_act(Xd, scale_dev=s_dev)
    acc = torch.zeros((T, O), dtype=torch.int32, device=DEV)
    y = torch.zeros((T, O), dtype=torch.float32, device=DEV)
    nm.nm_gemm(Xq, 0.0, *packed, O, N, M, bits, acc=acc, out=y, out_dtype=NM_OUT_F32, layout=TILED, act_scale_dev=s_dev)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    tol = 1e-5 * np.abs(acc_ref) * float(s_ref) * ref[2][None, :]
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - y_ref) <= tol + 1e-30)


# ---- which kernel variant a call launches -------------------------------------------------------

@pytest.mark.parametrize("T,K,O,N,M,bits,dtype,expect", [
    (4096, 768, 3072, 2, 4, 8, torch.bfloat16, {133}),          # BERT-base FFN-up and QKV: two 128 x 192 workgroups per CU
    (4096, 768, 2304, 2, 4, 8, torch.bfloat16, {133}),
    (4096, 768, 768, 2, 4, 8, torch.bfloat16, {116, 113}),      # the narrow outputs: 128 x 96
    (4096, 3072, 768, 2, 4, 8, torch.bfloat16, {116, 113}),
    (12288, 1024, 4096, 2, 4, 8, torch.bfloat16, {136}),        # BERT-large FFN-up: two 128 x 256 workgroups per CU
    (12288, 4096, 1024, 2, 4, 8, torch.bfloat16, {123}),        # long reduction: 256 x 256
    (49152, 768, 3072, 2, 4, 8, torch.bfloat16, {122, 123}),    # output larger than the Infinity Cache: no two-per-CU shape
    (4096, 768, 3072, 2, 8, 4, torch.bfloat16, {133}),          # a decoded pattern on a short reduction
    (4096, 768, 3072, 4, 4, 4, torch.bfloat16, {133}),          # dense int4
    (4096, 768, 3072, 4, 8, 4, torch.bfloat16, {126}),          # 4:8 int4 keeps 256 x 192 with the wavefronts 2 x 4
    (128, 768, 768, 2, 4, 8, torch.bfloat16, {130}),            # few tokens: the smallest tile
])
def test_tile_choice_on_the_paper_shapes(T, K, O, N, M, bits, dtype, expect):
    """The launcher's tile choice on the layer shapes the benchmarks run, read back through the measurement hook
    (timing-derived, so a change of it should be a decision, not an accident), and that the chosen kernel's output
    equals that of another tile variant on the same operands."""
    say("tile choice", T, K, O, N, M, bits)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(T + K + O)
    W = torch.randn((O, K), generator=gen, device=DEV, dtype=torch.float32) * 0.02
    X = torch.randint(-127, 128, (T, K), generator=gen, device=DEV, dtype=torch.int8)
    packed = nm.nm_compress(W, N, M, bits, layout=TILED)
    out = torch.zeros((T, O), dtype=dtype, device=DEV)
    nm.nm_gemm(X, 0.05, *packed, O, N, M, bits, out=out, out_dtype=NM_OUT_BF16, layout=TILED)
    tile = binding.raw().nm_bench_last_gemm_tile()
    torch.cuda.synchronize()
    assert tile in expect, "tile %d, expected one of %s" % (tile, sorted(expect))
    other = torch.zeros((T, O), dtype=dtype, device=DEV)
    with forced_tile(117 if tile != 117 else 116):
        nm.nm_gemm(X, 0.05, *packed, O, N, M, bits, out=other, out_dtype=NM_OUT_BF16, layout=TILED)
        torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), other.view(torch.int16))
