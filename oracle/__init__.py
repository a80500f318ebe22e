"""CPU oracle for the N:M-sparse low-bit integer path (test infrastructure only).

Thin numpy/ctypes front end over ``nm_oracle.c``; every piece of arithmetic
lives in the C file, which cites the passages of the paper it follows.  Only
the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nm_oracle.c")
_LIB = os.path.join(_HERE, "libnm_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.nmo_row_scale.restype = ctypes.c_float
        _lib.nmo_row_scale.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        _lib.nmo_quantize_one.restype = ctypes.c_int
        _lib.nmo_quantize_one.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_int]
        _lib.nmo_tiled_bytes.restype = ctypes.c_size_t
        _lib.nmo_tiled_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_size_t]
        _lib.nmo_to_tiled.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        _lib.nmo_from_tiled.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__("oracle returned %d" % code)
        self.code = code


def _check(rc: int):
    if rc != 0:
        raise OracleError(rc)


def _p(a):
    return None if a is None or a.size == 0 else ctypes.c_void_p(a.ctypes.data)


def num_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS or the core count)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def packed_sizes(rows, cols, N, M, bits):
    v, m, s = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(_load().nmo_packed_sizes(rows, cols, N, M, bits,
                                    ctypes.byref(v), ctypes.byref(m), ctypes.byref(s)))
    return v.value, m.value, s.value


def unit_bytes(N, M, bits):
    """(value bytes, index bytes) of the packed entries covering 32 input columns of one row."""
    epu = 32 // M * N
    ib = 0 if N >= M else (2 if M == 4 else 4)
    return epu * bits // 8, epu * ib // 8


def to_tiled(vals, meta, cols, N, M, bits):
    """Row layout -> tiled layout (both arrays; flat uint8).  A dense matrix has no metadata."""
    vals = np.ascontiguousarray(vals, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    rows = vals.shape[0]
    out = []
    for a, ub in zip((vals, meta), unit_bytes(N, M, bits)):
        if ub == 0:
            out.append(np.zeros(0, dtype=np.uint8))
            continue
        t = np.zeros(_load().nmo_tiled_bytes(rows, cols, ub), dtype=np.uint8)
        _check(_load().nmo_to_tiled(_p(a), rows, cols, ub, _p(t)))
        out.append(t)
    return out[0], out[1]


def from_tiled(vals_t, meta_t, rows, cols, N, M, bits):
    """Tiled layout -> row layout: (vals [rows, vstride], meta [rows, mstride])."""
    out = []
    for a, ub in zip((vals_t, meta_t), unit_bytes(N, M, bits)):
        r = np.zeros((rows, cols // 32 * ub), dtype=np.uint8)
        if ub:
            a = np.ascontiguousarray(a, dtype=np.uint8)
            assert a.size == _load().nmo_tiled_bytes(rows, cols, ub)
            _check(_load().nmo_from_tiled(_p(a), rows, cols, ub, _p(r)))
        out.append(r)
    return out[0], out[1]


def project(W, N, M):
    """Kept column offsets, shape [rows, cols/M, N], ascending inside a group."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    kept = np.zeros((rows, max(cols // M, 0), N), dtype=np.uint8)
    _check(_load().nmo_project(_p(W), rows, cols, cols, N, M, _p(kept)))
    return kept


def row_scale(w, bits):
    w = np.ascontiguousarray(w, dtype=np.float32)
    return np.float32(_load().nmo_row_scale(_p(w), w.shape[0], bits))


def quantize_one(w, s, bits):
    return int(_load().nmo_quantize_one(float(np.float32(w)), float(np.float32(s)), bits))


def compress(W, N, M, bits):
    """(vals uint8 [rows, vstride], meta uint8 [rows, mstride], scales float32 [rows])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    vb, mb, _ = packed_sizes(rows, cols, N, M, bits)
    vals = np.zeros((rows, vb // rows), dtype=np.uint8)
    meta = np.zeros((rows, mb // rows), dtype=np.uint8)
    scales = np.zeros(rows, dtype=np.float32)
    _check(_load().nmo_compress(_p(W), rows, cols, cols, N, M, bits,
                                _p(vals), _p(meta), _p(scales)))
    return vals, meta, scales


def compress_grouped(W, N, M, bits, rows_per_scale):
    """As compress, with one scale per group of rows_per_scale consecutive rows (scales is still
    float32 [rows]: every row's scale)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    vb, mb, _ = packed_sizes(rows, cols, N, M, bits)
    vals = np.zeros((rows, vb // rows), dtype=np.uint8)
    meta = np.zeros((rows, mb // rows), dtype=np.uint8)
    scales = np.zeros(rows, dtype=np.float32)
    _check(_load().nmo_compress_grouped(_p(W), rows, cols, cols, N, M, bits, rows_per_scale,
                                        _p(vals), _p(meta), _p(scales)))
    return vals, meta, scales


def dist_scales(W, N, M, bits, rows_per_scale, candidates):
    """(scales float32 [rows], errors float64 [groups, candidates/2 + 1]): the scale of every row's
    group that minimises the L2 distance between the kept weights and their quantised values."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    scales = np.zeros(rows, dtype=np.float32)
    ng = -(-rows // max(rows_per_scale, 1))
    errors = np.zeros((ng, max(candidates, 0) // 2 + 1), dtype=np.float64)
    _check(_load().nmo_dist_scales(_p(W), rows, cols, cols, N, M, bits, rows_per_scale, candidates, _p(scales), _p(errors)))
    return scales, errors


def compress_scaled(W, N, M, bits, scales):
    """(vals, meta): compress with the per-row scales given."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    rows, cols = W.shape
    vb, mb, _ = packed_sizes(rows, cols, N, M, bits)
    vals = np.zeros((rows, vb // rows), dtype=np.uint8)
    meta = np.zeros((rows, mb // rows), dtype=np.uint8)
    _check(_load().nmo_compress_scaled(_p(W), rows, cols, cols, N, M, bits, _p(scales), _p(vals), _p(meta)))
    return vals, meta


def decompress(vals, meta, rows, cols, N, M, bits):
    vals = np.ascontiguousarray(vals, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    Wq = np.zeros((rows, cols), dtype=np.int8)
    _check(_load().nmo_decompress(_p(vals), _p(meta), rows, cols, N, M, bits, _p(Wq)))
    return Wq


def gemm_sparse(X, vals, meta, O, N, M, bits):
    X = np.ascontiguousarray(X, dtype=np.int8)
    vals = np.ascontiguousarray(vals, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    T, K = X.shape
    acc = np.zeros((T, O), dtype=np.int32)
    _check(_load().nmo_gemm_sparse(_p(X), T, K, K, _p(vals), _p(meta), O, N, M, bits, _p(acc), O))
    return acc


def gemm_dense(X, Wq):
    X = np.ascontiguousarray(X, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    T, K = X.shape
    O = Wq.shape[0]
    acc = np.zeros((T, O), dtype=np.int32)
    _check(_load().nmo_gemm_dense(_p(X), T, K, K, _p(Wq), O, _p(acc), O))
    return acc


def dequant(acc, act_scale, scales, bias=None):
    """(fp32 output, bf16 output as uint16 bit patterns), both [tokens, O]."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    T, O = acc.shape
    f32 = np.zeros((T, O), dtype=np.float32)
    b16 = np.zeros((T, O), dtype=np.uint16)
    _check(_load().nmo_dequant(_p(acc), T, O, O, ctypes.c_float(act_scale), _p(scales), _p(bias),
                               _p(f32), _p(b16), O))
    return f32, b16


def requant(acc, act_scale, scales, out_scale, bias=None):
    """(int8 output [tokens, O], max |y|): the layer output quantised for the next layer."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    T, O = acc.shape
    q = np.zeros((T, O), dtype=np.int8)
    amax = ctypes.c_float(0.0)
    _check(_load().nmo_requant(_p(acc), T, O, O, ctypes.c_float(act_scale), _p(scales), _p(bias),
                               ctypes.c_float(out_scale), _p(q), O, ctypes.byref(amax)))
    return q, float(amax.value)


def quantize_act(X, scale=None):
    """(int8 codes [tokens, K], float32 scale): the per-tensor 8-bit activation quantiser; scale None =
    the largest magnitude / 127 (1 for an all-zero tensor)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    tokens, K = X.shape
    Q = np.empty((tokens, K), np.int8)
    s = ctypes.c_float(0.0)
    _check(_load().nmo_quantize_act(_p(X), tokens, K, K, ctypes.c_float(0.0 if scale is None else float(np.float32(scale))),
                                    _p(Q), K, ctypes.byref(s)))
    return Q, np.float32(s.value)


def admm_project(W, U, N, M, bits, rows_per_scale):
    """(Z, U_out, scales): the Z-update Z = Pi(W + U) with both constraints and the dual update
    U + W - Z; bits = 0 leaves the quantisation constraint out (scales is then None)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    if U is not None:
        U = np.ascontiguousarray(U, dtype=np.float32)
        assert U.shape == W.shape
    rows, cols = W.shape
    Z = np.zeros((rows, cols), dtype=np.float32)
    Uo = np.zeros((rows, cols), dtype=np.float32)
    scales = np.zeros(rows, dtype=np.float32) if bits else None
    _check(_load().nmo_admm_project(_p(W), _p(U), rows, cols, cols, N, M, bits, rows_per_scale,
                                    _p(Z), _p(Uo), cols, _p(scales)))
    return Z, Uo, scales
