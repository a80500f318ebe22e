"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, sizes buffers like the oracle, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2206_15014_amd as nm
from paper_2206_15014_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "nm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(nm_[a-z0-9_]+)\s*\(", header))
    assert names >= {"nm_packed_sizes", "nm_compress", "nm_compress_grouped", "nm_compress_batch", "nm_decompress_i8", "nm_gemm", "nm_gemm_q8",
                     "nm_gemm_batch", "nm_project", "nm_absmax_to_scale", "nm_absmax_f32", "nm_quantize_act", "nm_scale_search", "nm_scale_search_workspace_bytes", "nm_scale_search_static", "nm_compress_scaled", "nm_repack",
                     "nm_status_string"}
    lib = ctypes.CDLL(binding.library_path())
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("N,M,bits", [(2, 4, 8), (1, 4, 4), (2, 8, 4), (3, 4, 8), (7, 8, 4), (1, 8, 8), (4, 4, 8), (8, 8, 4)])
def test_sizes_agree_with_oracle(N, M, bits):
    for rows, cols in [(768, 768), (3072, 768), (1, M), (5, 3 * M), (1024, 4096)]:
        assert nm.nm_packed_sizes(rows, cols, N, M, bits) == oracle.packed_sizes(rows, cols, N, M, bits)
    # tiled layout: rows padded to a multiple of 16; the oracle's converter says how many bytes that is
    import numpy as np
    for rows, cols in [(768, 768), (5, 128), (130, 1024)]:
        v, m, _ = oracle.compress(np.zeros((rows, cols), np.float32), N, M, bits)
        vt, mt = oracle.to_tiled(v, m, cols, N, M, bits)
        assert nm.nm_packed_sizes(rows, cols, N, M, bits, binding.NM_LAYOUT_TILED) == (vt.size, mt.size, rows * 4)


def test_bad_patterns_are_rejected():
    for args, code in [((0, 8, 2, 4, 8), -2), ((8, 0, 2, 4, 8), -2), ((8, 8, 0, 4, 8), -3), ((8, 8, 5, 4, 8), -3),
                       ((8, 8, 2, 5, 8), -3), ((8, 10, 2, 4, 8), -3), ((8, 8, 2, 4, 6), -4), ((8, 8, 2, 16, 8), -3),
                       ((8, 8, 2, 4, 8, 2), -8), ((8, 8, 2, 4, 8, -1), -8), ((8, 64, 2, 4, 8, 1), -3)]:
        with pytest.raises(nm.NMError) as e:
            nm.nm_packed_sizes(*args)
        assert e.value.code == code
    assert nm.nm_packed_sizes(8, 8, 4, 4, 8) == (64, 0, 32)       # dense: no metadata


def test_entry_points_validate_before_launch():
    lib = binding.raw()
    P = 0x1000          # never dereferenced on the host; validation fails first
    assert lib.nm_compress(None, 8, 8, 8, 2, 4, 8, 0, P, P, P, None) == -1
    assert lib.nm_compress(P, 8, 8, 4, 2, 4, 8, 0, P, P, P, None) == -2          # ldw < cols
    assert lib.nm_compress(P, 8, 8, 8, 2, 4, 5, 0, P, P, P, None) == -4
    assert lib.nm_compress(P + 2, 8, 8, 8, 2, 4, 8, 0, P, P, P, None) == -6
    assert lib.nm_compress(P, 8, 8, 8, 2, 4, 8, 7, P, P, P, None) == -8          # unknown layout
    assert lib.nm_compress(P, 8, 8, 8, 2, 4, 8, 1, P, P, P, None) == -3          # tiled layout needs cols % 128 == 0
    assert lib.nm_compress(P, 8, 8, 8, 2, 4, 8, 0, P, None, P, None) == -1       # metadata buffer missing ...
    assert lib.nm_compress(P, 8, 8, 8, 4, 4, 8, 0, None, None, P, None) == -1    # ... which only a dense matrix may leave out
    assert lib.nm_decompress_i8(P, None, 8, 8, 2, 4, 8, 0, P, None) == -1
    assert lib.nm_compress_grouped(P, 8, 8, 8, 2, 4, 8, 0, 0, P, P, P, None) == -2   # rows_per_scale < 1
    assert lib.nm_compress_grouped(P, 8, 8, 8, 2, 4, 8, 0, 32, P, None, P, None) == -1
    assert lib.nm_compress_grouped(P, 8, 8, 8, 2, 4, 3, 0, 32, P, P, P, None) == -4
    Item = binding.CompressItem
    items = (Item * 2)(Item(P, 8, 8, 8, P, P, P), Item(P, 8, 16, 16, P, P, P))
    assert lib.nm_compress_batch(items, 0, 2, 4, 8, 0, None) == -2               # no items
    assert lib.nm_compress_batch(None, 2, 2, 4, 8, 0, None) == -1
    assert lib.nm_compress_batch(items, 65537, 2, 4, 8, 0, None) == -2           # more items than a call takes
    assert lib.nm_compress_batch(items, 2, 2, 4, 7, 0, None) == -4
    assert lib.nm_compress_batch(items, 2, 2, 4, 8, 1, None) == -3               # tiled layout, widths not multiples of 128
    for bad, code in [(Item(None, 8, 8, 8, P, P, P), -1), (Item(P, 8, 8, 8, P, None, P), -1), (Item(P, 8, 8, 4, P, P, P), -2),
                      (Item(P, 0, 8, 8, P, P, P), -2), (Item(P, 8, 10, 12, P, P, P), -3), (Item(P + 2, 8, 8, 8, P, P, P), -6)]:
        arr = (Item * 2)(items[0], bad)                                       # a bad item anywhere refuses the whole call
        assert lib.nm_compress_batch(arr, 2, 2, 4, 8, 0, None) == code
    g = lambda **k: lib.nm_gemm(*[k.get(n, d) for n, d in [
        ("X", P), ("T", 4), ("K", 8), ("ldx", 8), ("s", 1.0), ("sd", None), ("v", P), ("m", P), ("sc", P), ("O", 8), ("N", 2),
        ("M", 4), ("bits", 8), ("layout", 0), ("bias", None), ("acc", P), ("out", None), ("dt", 0), ("ldo", 8), ("st", None)]])
    assert g(X=None) == -1
    assert g(T=0) == -2
    assert g(ldx=4) == -2
    assert g(ldo=4) == -2
    assert g(N=5) == -3
    assert g(K=6) == -3
    assert g(bits=16) == -4
    assert g(layout=3) == -8
    assert g(layout=1) == -3                 # K % 128 != 0
    assert g(m=None) == -1 and g(m=None, N=4, X=None) == -1   # a dense matrix needs no metadata (the call gets as far as the next check)
    assert g(dt=3, out=P) == -5
    assert g(dt=1) == -5                     # dtype set but no output buffer
    assert g(out=P) == -5                    # output buffer but dtype none
    assert g(acc=None) == -1                 # nothing to write
    assert g(acc=P + 1) == -6
    assert g(sd=P + 2) == -6
    pj = lambda **k: lib.nm_project(*[k.get(n, d) for n, d in [
        ("W", P), ("U", None), ("rows", 8), ("cols", 8), ("ldw", 8), ("N", 2), ("M", 4), ("bits", 8), ("rps", 32),
        ("Z", P), ("Uo", None), ("ldz", 8), ("sc", P), ("st", None)]])
    assert pj(W=None) == -1 and pj(Z=None) == -1
    assert pj(sc=None) == -1                 # scales are required with a quantisation constraint ...
    assert pj(sc=None, bits=0, W=None) == -1 # ... and not without one (the call gets as far as the next check)
    assert pj(rps=0) == -2 and pj(ldz=4) == -2 and pj(ldw=4) == -2
    assert pj(N=5) == -3 and pj(cols=6) == -3
    assert pj(bits=5) == -4
    assert pj(W=P + 4) == -6 and pj(Uo=P + 8) == -6 and pj(ldw=10, cols=8) == -6
    q = lambda **k: lib.nm_gemm_q8(*[k.get(n, d) for n, d in [
        ("X", P), ("T", 4), ("K", 8), ("ldx", 8), ("s", 1.0), ("sd", None), ("v", P), ("m", P), ("sc", P), ("O", 8), ("N", 2),
        ("M", 4), ("bits", 8), ("layout", 0), ("bias", None), ("so", 0.5), ("sod", None), ("out", P), ("ldo", 8), ("amax", None), ("st", None)]])
    assert q(out=None) == -1
    assert q(X=None) == -1
    assert q(T=0) == -2
    assert q(ldo=4) == -2
    assert q(N=5) == -3
    assert q(bits=5) == -4
    assert q(so=0.0) == -9 and q(so=-1.0) == -9 and q(so=float("inf")) == -9 and q(so=float("nan")) == -9
    assert q(so=0.0, sod=P, X=None) == -1    # with a device scale the host value is not looked at
    assert q(out=P + 2) == -6
    assert q(amax=P + 1) == -6
    assert q(sod=P + 1) == -6
    lib.nm_scale_search_workspace_bytes.restype = ctypes.c_size_t
    assert lib.nm_scale_search_workspace_bytes(768, 32) == 768 * 17 * 8
    assert lib.nm_scale_search_workspace_bytes(768, 33) == 0 and lib.nm_scale_search_workspace_bytes(0, 32) == 0
    ss = lambda **k: lib.nm_scale_search(*[k.get(n, d) for n, d in [
        ("W", P), ("rows", 8), ("cols", 8), ("ldw", 8), ("N", 2), ("M", 4), ("bits", 8), ("rps", 4), ("C", 16), ("sc", P),
        ("ws", P), ("wsb", 8 * 9 * 8), ("st", None)]])
    assert ss(W=None) == -1 and ss(sc=None) == -1 and ss(ws=None) == -1
    assert ss(C=0) == -2 and ss(C=7) == -2 and ss(C=66) == -2 and ss(rps=0) == -2 and ss(ldw=4) == -2
    assert ss(N=5) == -3 and ss(bits=3) == -4
    assert ss(ws=P + 4) == -6 and ss(W=P + 1) == -6
    assert ss(wsb=8 * 9 * 8 - 1) == -10
    cs = lambda **k: lib.nm_compress_scaled(*[k.get(n, d) for n, d in [
        ("W", P), ("rows", 8), ("cols", 8), ("ldw", 8), ("N", 2), ("M", 4), ("bits", 8), ("layout", 0), ("sc", P), ("v", P), ("m", P), ("st", None)]])
    assert cs(sc=None) == -1 and cs(v=None) == -1 and cs(m=None) == -1 and cs(m=None, N=4, W=None) == -1
    assert cs(ldw=4) == -2 and cs(layout=1) == -3 and cs(layout=5) == -8 and cs(sc=P + 2) == -6
    assert lib.nm_repack(P, P, 8, 8, 2, 4, 8, 0, P, P, None) == -3          # cols % 128
    assert lib.nm_repack(P, None, 8, 128, 2, 4, 8, 0, P, P, None) == -1 and lib.nm_repack(P, P, 8, 128, 2, 4, 8, 2, P, P, None) == -8
    assert lib.nm_repack(None, None, 8, 128, 4, 4, 8, 1, P, None, None) == -1
    assert lib.nm_absmax_to_scale(None, P, 0, None) == -1 and lib.nm_absmax_to_scale(P, None, 0, None) == -1
    assert lib.nm_absmax_to_scale(P, P + 2, 0, None) == -6
    assert lib.nm_absmax_to_scale(P, P, 0, None) == -2
    assert lib.nm_absmax_f32(None, 4, 8, 8, P, None) == -1 and lib.nm_absmax_f32(P, 4, 8, 8, None, None) == -1
    assert lib.nm_absmax_f32(P, 0, 8, 8, P, None) == -2 and lib.nm_absmax_f32(P, 4, 0, 8, P, None) == -2 and lib.nm_absmax_f32(P, 4, 8, 7, P, None) == -2
    assert lib.nm_absmax_f32(P + 2, 4, 8, 8, P, None) == -6 and lib.nm_absmax_f32(P, 4, 8, 8, P + 1, None) == -6
    qa = lambda **k: lib.nm_quantize_act(*[k.get(n, d) for n, d in [
        ("X", P), ("T", 4), ("K", 8), ("ldx", 8), ("s", ctypes.c_float(0.5)), ("sd", None), ("Q", P), ("ldq", 8), ("st", None)]])
    assert qa(X=None) == -1 and qa(Q=None) == -1
    assert qa(T=0) == -2 and qa(K=-1) == -2 and qa(ldx=7) == -2 and qa(ldq=7) == -2
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        assert qa(s=ctypes.c_float(bad)) == -9
    assert qa(X=P + 1) == -6 and qa(sd=P + 2) == -6


def test_status_strings():
    assert nm.nm_status_string(0) == "ok"
    assert all(nm.nm_status_string(c) not in ("", "unknown status") for c in range(-10, 1))
    assert nm.nm_status_string(-99) == "unknown status"


def test_gemm_batch_validates_before_launch():
    lib = binding.raw()
    P = 0x1000          # never dereferenced on the host; validation fails first
    item = lambda **k: binding.GemmItem(*[k.get(n, d) for n, d in [
        ("X", P), ("tokens", 4), ("K", 8), ("ldx", 8), ("act_scale", 1.0), ("act_scale_dev", None), ("vals", P), ("meta", P),
        ("scales", P), ("O", 8), ("bias", None), ("acc", P), ("out", None), ("ldo", 8)]])
    call = lambda items, count=None, N=2, M=4, bits=8, layout=0, out_dtype=0: lib.nm_gemm_batch(
        (binding.GemmItem * max(len(items), 1))(*items), len(items) if count is None else count, N, M, bits, layout, out_dtype, None)
    assert lib.nm_gemm_batch(None, 1, 2, 4, 8, 0, 0, None) == -1
    assert call([item()], count=0) == -2
    assert call([item()] * 5) == -2                              # more than NM_GEMM_BATCH_MAX_ITEMS
    assert call([item()], out_dtype=3) == -5
    assert call([item(), item(X=None)]) == -1                    # the second item is refused: nothing is enqueued
    assert call([item(), item(ldo=4)]) == -2
    assert call([item(), item(acc=None)]) == -1                  # no output at all
    assert call([item(out=P)]) == -5                             # output given, output type none
    assert call([item(), item(acc=P + 2)]) == -6
    assert call([item()], N=5) == -3
    assert call([item()], bits=5) == -4
    assert call([item()], layout=9) == -8
    assert call([item()], layout=1) == -3                        # tiled layout needs K % 128 == 0
