"""ctypes binding of libnm (declared in include/nm.h): argument marshalling only.

Tensors are torch CUDA tensors used purely as device buffers; the current torch
stream is handed to the library.  There is no CPU fallback: a missing library is
an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnm.so")

NM_OUT_NONE, NM_OUT_F32, NM_OUT_BF16 = 0, 1, 2
NM_LAYOUT_ROWS, NM_LAYOUT_TILED = 0, 1


class CompressItem(ctypes.Structure):
    """nm_compress_item of include/nm.h."""
    _fields_ = [("W_dev", ctypes.c_void_p), ("rows", ctypes.c_int), ("cols", ctypes.c_int), ("ldw", ctypes.c_int),
                ("vals_dev", ctypes.c_void_p), ("meta_dev", ctypes.c_void_p), ("scales_dev", ctypes.c_void_p)]


class GemmItem(ctypes.Structure):
    """nm_gemm_item of include/nm.h."""
    _fields_ = [("X_dev", ctypes.c_void_p), ("tokens", ctypes.c_int), ("K", ctypes.c_int), ("ldx", ctypes.c_int),
                ("act_scale", ctypes.c_float), ("act_scale_dev", ctypes.c_void_p),
                ("vals_dev", ctypes.c_void_p), ("meta_dev", ctypes.c_void_p), ("scales_dev", ctypes.c_void_p), ("O", ctypes.c_int),
                ("bias_dev", ctypes.c_void_p), ("acc_dev", ctypes.c_void_p), ("out_dev", ctypes.c_void_p), ("ldo", ctypes.c_int)]


_lib = None


class NMError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__("%s failed: %s (%d)" % (where, nm_status_string(code), code))
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libnm.so is not built (%s); run `python -c 'import __graft_entry__ as g; g.build()'`"
            % _LIB_PATH)
    # torch first: the process must hold ONE HIP runtime, and torch brings its own copy; with it
    # already loaded, libnm's dependency on libamdhip64 resolves to that same copy.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    c_int, c_vp, c_f = ctypes.c_int, ctypes.c_void_p, ctypes.c_float
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.nm_packed_sizes.restype = c_int
    lib.nm_packed_sizes.argtypes = [c_int] * 6 + [szp] * 3
    lib.nm_compress.restype = c_int
    lib.nm_compress.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp]
    lib.nm_compress_grouped.restype = c_int
    lib.nm_compress_grouped.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp]
    lib.nm_compress_batch.argtypes = [ctypes.POINTER(CompressItem), c_int, c_int, c_int, c_int, c_int, c_vp]
    lib.nm_compress_batch.restype = c_int
    lib.nm_decompress_i8.restype = c_int
    lib.nm_decompress_i8.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp]
    lib.nm_gemm.restype = c_int
    lib.nm_gemm.argtypes = [c_vp, c_int, c_int, c_int, c_f, c_vp, c_vp, c_vp, c_vp,
                            c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_int, c_int, c_vp]
    lib.nm_gemm_batch.restype = c_int
    lib.nm_gemm_batch.argtypes = [ctypes.POINTER(GemmItem), c_int, c_int, c_int, c_int, c_int, c_int, c_vp]
    lib.nm_compress_scaled.restype = c_int
    lib.nm_compress_scaled.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp]
    lib.nm_scale_search_workspace_bytes.restype = ctypes.c_size_t
    lib.nm_scale_search_workspace_bytes.argtypes = [c_int, c_int]
    lib.nm_scale_search.restype = c_int
    lib.nm_scale_search.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, ctypes.c_size_t, c_vp]
    lib.nm_scale_search_static.restype = c_int
    lib.nm_scale_search_static.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp]
    lib.nm_repack.restype = c_int
    lib.nm_repack.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp]
    lib.nm_project.restype = c_int
    lib.nm_project.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_int, c_vp, c_vp]
    lib.nm_gemm_q8.restype = c_int
    lib.nm_gemm_q8.argtypes = [c_vp, c_int, c_int, c_int, c_f, c_vp, c_vp, c_vp, c_vp,
                               c_int, c_int, c_int, c_int, c_int, c_vp, c_f, c_vp, c_vp, c_int, c_vp, c_vp]
    lib.nm_absmax_to_scale.restype = c_int
    lib.nm_absmax_to_scale.argtypes = [c_vp, c_vp, c_int, c_vp]
    lib.nm_absmax_f32.restype = c_int
    lib.nm_absmax_f32.argtypes = [c_vp, c_int, c_int, c_int, c_vp, c_vp]
    lib.nm_quantize_act.restype = c_int
    lib.nm_quantize_act.argtypes = [c_vp, c_int, c_int, c_int, c_f, c_vp, c_vp, c_int, c_vp]
    lib.nm_test_force_gemm_tile.restype = c_int
    lib.nm_test_force_gemm_tile.argtypes = [c_int]
    lib.nm_bench_last_gemm_tile.restype = c_int
    lib.nm_bench_last_gemm_tile.argtypes = []
    lib.nm_bench_smfmac_probe.restype = c_int
    lib.nm_bench_smfmac_probe.argtypes = [c_int, c_int, c_vp, c_vp]
    lib.nm_status_string.restype = ctypes.c_char_p
    lib.nm_status_string.argtypes = [c_int]
    _lib = lib
    return lib


def raw():
    """The loaded ctypes library (for callers that marshal pointers themselves)."""
    return _load()


def nm_status_string(status: int) -> str:
    return _load().nm_status_string(int(status)).decode()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def force_gemm_tile(cfg: int) -> int:
    """Test hook (not part of the ABI): force the tile variant nm_gemm launches; 0 = automatic."""
    return _load().nm_test_force_gemm_tile(int(cfg))


def nm_packed_sizes(rows: int, cols: int, N: int, M: int, bits: int, layout: int = NM_LAYOUT_ROWS) -> Tuple[int, int, int]:
    v, m, s = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    rc = _load().nm_packed_sizes(rows, cols, N, M, bits, layout, ctypes.byref(v), ctypes.byref(m), ctypes.byref(s))
    if rc:
        raise NMError(rc, "nm_packed_sizes")
    return v.value, m.value, s.value


def _packed_buffers(rows, cols, N, M, bits, layout, device, vals, meta, scales):
    """The three output buffers of a compress call: [rows, stride] in the row layout, flat in the tiled one."""
    import torch
    vb, mb, _ = nm_packed_sizes(rows, cols, N, M, bits, layout)
    shape = (lambda nbytes: (rows, nbytes // rows)) if layout == NM_LAYOUT_ROWS else (lambda nbytes: (nbytes,))
    if vals is None:
        vals = torch.empty(shape(vb), dtype=torch.uint8, device=device)
    if meta is None:
        meta = torch.empty(shape(mb), dtype=torch.uint8, device=device)
    if scales is None:
        scales = torch.empty(rows, dtype=torch.float32, device=device)
    return vals, meta, scales


def nm_compress(W, N: int, M: int, bits: int, vals=None, meta=None, scales=None, stream=None, layout: int = NM_LAYOUT_ROWS):
    """W: float32 CUDA tensor [rows, cols] (row stride may exceed cols).

    Returns (vals uint8, meta uint8, scales float32 [rows]); vals / meta are [rows, stride] in the
    row layout and flat in the tiled one.
    """
    rows, cols = W.shape
    vals, meta, scales = _packed_buffers(rows, cols, N, M, bits, layout, W.device, vals, meta, scales)
    rc = _load().nm_compress(_ptr(W), rows, cols, W.stride(0), N, M, bits, layout,
                             _ptr(vals), _ptr(meta), _ptr(scales), _stream(stream))
    if rc:
        raise NMError(rc, "nm_compress")
    return vals, meta, scales


def nm_compress_grouped(W, N: int, M: int, bits: int, rows_per_scale: int, vals=None, meta=None, scales=None, stream=None,
                        layout: int = NM_LAYOUT_ROWS):
    """As nm_compress, with one scale per group of rows_per_scale consecutive rows; scales is
    still float32 [rows] (the rows of a group hold the same value)."""
    rows, cols = W.shape
    vals, meta, scales = _packed_buffers(rows, cols, N, M, bits, layout, W.device, vals, meta, scales)
    rc = _load().nm_compress_grouped(_ptr(W), rows, cols, W.stride(0), N, M, bits, layout, rows_per_scale,
                                     _ptr(vals), _ptr(meta), _ptr(scales), _stream(stream))
    if rc:
        raise NMError(rc, "nm_compress_grouped")
    return vals, meta, scales


def nm_scale_search(W, N: int, M: int, bits: int, rows_per_scale: int, candidates: int, scales=None, workspace=None, stream=None):
    """The distance-minimising scale of every row's group (float32 [rows]); workspace: uint8 CUDA tensor of
    nm_scale_search_workspace_bytes(rows, candidates) bytes, allocated here when not given."""
    import torch
    rows, cols = W.shape
    if scales is None:
        scales = torch.empty(rows, dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = torch.empty(max(_load().nm_scale_search_workspace_bytes(rows, candidates), 8), dtype=torch.uint8, device=W.device)
    rc = _load().nm_scale_search(_ptr(W), rows, cols, W.stride(0), N, M, bits, rows_per_scale, candidates, _ptr(scales),
                                 _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise NMError(rc, "nm_scale_search")
    return scales


def nm_scale_search_static(W, N: int, M: int, bits: int, rows_per_scale: int, candidates: int, scales, stream=None):
    """nm_scale_search on the library's built-in scratch array: allocates nothing, so `scales` (float32 [rows]) must be given."""
    rows, cols = W.shape
    rc = _load().nm_scale_search_static(_ptr(W), rows, cols, W.stride(0), N, M, bits, rows_per_scale, candidates, _ptr(scales), _stream(stream))
    if rc:
        raise NMError(rc, "nm_scale_search_static")
    return scales


def nm_compress_scaled(W, N: int, M: int, bits: int, scales, vals=None, meta=None, stream=None, layout: int = NM_LAYOUT_ROWS):
    """nm_compress with the per-row scales given (float32 CUDA tensor [rows]); returns (vals, meta, scales)."""
    rows, cols = W.shape
    vals, meta, scales = _packed_buffers(rows, cols, N, M, bits, layout, W.device, vals, meta, scales)
    rc = _load().nm_compress_scaled(_ptr(W), rows, cols, W.stride(0), N, M, bits, layout, _ptr(scales),
                                    _ptr(vals), _ptr(meta), _stream(stream))
    if rc:
        raise NMError(rc, "nm_compress_scaled")
    return vals, meta, scales


def compress_items(Ws, outs):
    """The nm_compress_item array for matrices Ws and their (vals, meta, scales) buffers."""
    arr = (CompressItem * len(Ws))()
    for i, (W, (vals, meta, scales)) in enumerate(zip(Ws, outs)):
        rows, cols = W.shape
        arr[i] = CompressItem(_ptr(W), rows, cols, W.stride(0), _ptr(vals), _ptr(meta), _ptr(scales))
    return arr


def nm_compress_batch(Ws, N: int, M: int, bits: int, outs=None, stream=None, layout: int = NM_LAYOUT_ROWS):
    """nm_compress of every matrix of the list Ws (float32 CUDA tensors [rows, cols]) in one call.

    Returns the list of (vals, meta, scales), one per matrix, as nm_compress would.
    """
    if outs is None:
        outs = [_packed_buffers(W.shape[0], W.shape[1], N, M, bits, layout, W.device, None, None, None) for W in Ws]
    arr = compress_items(Ws, outs)
    rc = _load().nm_compress_batch(arr, len(Ws), N, M, bits, layout, _stream(stream))
    if rc:
        raise NMError(rc, "nm_compress_batch")
    return outs


def nm_repack(vals, meta, rows: int, cols: int, N: int, M: int, bits: int, layout_in: int, stream=None):
    """(vals, meta) in the other layout than layout_in (a byte permutation; the scales do not change)."""
    layout_out = NM_LAYOUT_TILED if layout_in == NM_LAYOUT_ROWS else NM_LAYOUT_ROWS
    v, m, _ = _packed_buffers(rows, cols, N, M, bits, layout_out, vals.device, None, None, 0)
    rc = _load().nm_repack(_ptr(vals), _ptr(meta), rows, cols, N, M, bits, layout_in, _ptr(v), _ptr(m), _stream(stream))
    if rc:
        raise NMError(rc, "nm_repack")
    return v, m


def nm_decompress_i8(vals, meta, rows: int, cols: int, N: int, M: int, bits: int, out=None, stream=None,
                     layout: int = NM_LAYOUT_ROWS):
    import torch
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.int8, device=vals.device)
    rc = _load().nm_decompress_i8(_ptr(vals), _ptr(meta), rows, cols, N, M, bits, layout, _ptr(out), _stream(stream))
    if rc:
        raise NMError(rc, "nm_decompress_i8")
    return out


def nm_gemm(X, act_scale: float, vals, meta, scales, O: int, N: int, M: int, bits: int,
            bias=None, acc=None, out=None, out_dtype: int = NM_OUT_NONE, ldo: Optional[int] = None,
            stream=None, layout: int = NM_LAYOUT_ROWS, act_scale_dev=None):
    """X: int8 CUDA tensor [tokens, K].  acc (int32) and out (float32 / bfloat16), when
    given, are [tokens, ldo] buffers written in place; returns (acc, out)."""
    tokens, K = X.shape
    if ldo is None:
        ref = out if out is not None else acc
        ldo = ref.stride(0) if ref is not None and hasattr(ref, "stride") else O
    rc = _load().nm_gemm(_ptr(X), tokens, K, X.stride(0), float(act_scale), _ptr(act_scale_dev),
                         _ptr(vals), _ptr(meta), _ptr(scales), O, N, M, bits, layout,
                         _ptr(bias), _ptr(acc), _ptr(out), out_dtype, ldo, _stream(stream))
    if rc:
        raise NMError(rc, "nm_gemm")
    return acc, out


def gemm_items(calls):
    """The nm_gemm_item array for `calls`: dicts with X, act_scale, vals, meta, scales, O and, optionally,
    bias, acc, out, ldo, act_scale_dev (the arguments of nm_gemm with the same names)."""
    arr = (GemmItem * len(calls))()
    for i, c in enumerate(calls):
        X = c["X"]
        tokens, K = X.shape
        ref = c.get("out") if c.get("out") is not None else c.get("acc")
        ldo = c.get("ldo")
        if ldo is None:
            ldo = ref.stride(0) if ref is not None else c["O"]
        arr[i] = GemmItem(_ptr(X), tokens, K, X.stride(0), float(c["act_scale"]), _ptr(c.get("act_scale_dev")),
                          _ptr(c["vals"]), _ptr(c.get("meta")), _ptr(c["scales"]), c["O"],
                          _ptr(c.get("bias")), _ptr(c.get("acc")), _ptr(c.get("out")), ldo)
    return arr


def nm_gemm_batch(calls, N: int, M: int, bits: int, out_dtype: int = NM_OUT_NONE, stream=None, layout: int = NM_LAYOUT_ROWS):
    """nm_gemm for every entry of `calls` (see gemm_items) in one call; outputs are written in place."""
    arr = gemm_items(calls)
    rc = _load().nm_gemm_batch(arr, len(calls), N, M, bits, layout, out_dtype, _stream(stream))
    if rc:
        raise NMError(rc, "nm_gemm_batch")


def nm_gemm_q8(X, act_scale: float, vals, meta, scales, O: int, N: int, M: int, bits: int,
               out_scale: float, out, bias=None, absmax=None, ldo: Optional[int] = None, stream=None,
               layout: int = NM_LAYOUT_ROWS, act_scale_dev=None, out_scale_dev=None):
    """X: int8 CUDA tensor [tokens, K]; out: int8 [tokens, ldo] written in place with the layer's
    output as 8-bit codes of scale out_scale; absmax: optional float32 tensor of one element,
    max |y| is max-combined into it.  act_scale_dev / out_scale_dev: optional float32 tensors of
    one element that replace the host values.  Returns out."""
    tokens, K = X.shape
    if ldo is None:
        ldo = out.stride(0)
    rc = _load().nm_gemm_q8(_ptr(X), tokens, K, X.stride(0), float(act_scale), _ptr(act_scale_dev),
                            _ptr(vals), _ptr(meta), _ptr(scales), O, N, M, bits, layout,
                            _ptr(bias), float(out_scale), _ptr(out_scale_dev), _ptr(out), ldo, _ptr(absmax), _stream(stream))
    if rc:
        raise NMError(rc, "nm_gemm_q8")
    return out


def nm_absmax_to_scale(absmax, scale, reset: bool = False, stream=None):
    """scale[0] = absmax[0] / 127 (1 when it is 0) on the stream; reset: absmax[0] = 0 afterwards."""
    rc = _load().nm_absmax_to_scale(_ptr(absmax), _ptr(scale), int(bool(reset)), _stream(stream))
    if rc:
        raise NMError(rc, "nm_absmax_to_scale")
    return scale


def nm_absmax_f32(X, absmax, stream=None):
    """X: float32 CUDA tensor [tokens, K] (row stride >= K); absmax: float32 tensor of one element
    that the caller has set (0, or a running maximum): max |X| is max-combined into it.  Returns
    absmax."""
    tokens, K = X.shape
    rc = _load().nm_absmax_f32(_ptr(X), tokens, K, X.stride(0), _ptr(absmax), _stream(stream))
    if rc:
        raise NMError(rc, "nm_absmax_f32")
    return absmax


def nm_quantize_act(X, scale: float = 0.0, out=None, scale_dev=None, stream=None):
    """X: float32 CUDA tensor [tokens, K] -> int8 codes clamp(rne(X / s), -127, 127) with the
    tensor's one scale s: `scale`, or the float32 tensor of one element `scale_dev` that
    replaces it.  `out` (int8 [tokens, >= K] by row stride) is allocated here when not passed.
    Returns out."""
    import torch
    tokens, K = X.shape
    if out is None:
        out = torch.empty((tokens, K), dtype=torch.int8, device=X.device)
    rc = _load().nm_quantize_act(_ptr(X), tokens, K, X.stride(0), float(scale), _ptr(scale_dev),
                                 _ptr(out), out.stride(0), _stream(stream))
    if rc:
        raise NMError(rc, "nm_quantize_act")
    return out


def nm_project(W, U, N: int, M: int, bits: int, rows_per_scale: int, Z=None, U_out=None, scales=None, stream=None):
    """W, U (or None): float32 CUDA tensors [rows, cols].  Returns (Z, U_out, scales): the ADMM
    Z-update Z = Pi(W + U) with both constraints (bits = 0: sparsity only, scales is then None)
    and the dual update U + W - Z.  Buffers that are not passed are allocated here."""
    import torch
    rows, cols = W.shape
    if Z is None:
        Z = torch.empty((rows, cols), dtype=torch.float32, device=W.device)
    if U_out is None:
        U_out = torch.empty((rows, cols), dtype=torch.float32, device=W.device)
    if scales is None and bits:
        scales = torch.empty(rows, dtype=torch.float32, device=W.device)
    if U is not None and U.stride(0) != W.stride(0):
        raise ValueError("W and U must share their leading dimension")
    if U_out.stride(0) != Z.stride(0):
        raise ValueError("Z and U_out must share their leading dimension")
    rc = _load().nm_project(_ptr(W), _ptr(U), rows, cols, W.stride(0), N, M, bits, rows_per_scale,
                            _ptr(Z), _ptr(U_out), Z.stride(0), _ptr(scales), _stream(stream))
    if rc:
        raise NMError(rc, "nm_project")
    return Z, U_out, scales
