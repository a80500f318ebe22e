"""The entry point that allocates nothing (nm_scale_search_static, scratch in a static device array of the
library) against the entry point it is a variant of (nm_scale_search, scratch in a caller's workspace):
the same scales bit for bit, called through the raw C ABI, on two calls in a row of which the second works
on a smaller matrix (what the first call left in the array must not matter); sizes beyond the array are
refused before anything is enqueued."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2206_15014_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(lib, W, N, M, bits, rps, C):
    rows, cols = W.shape
    Wd = torch.from_numpy(W).to(DEV)
    st = torch.cuda.current_stream().cuda_stream
    need = lib.nm_scale_search_workspace_bytes(rows, C)
    ws = torch.full((need,), 0xEE, dtype=torch.uint8, device=DEV)
    s_ws = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    s_st = torch.full((rows,), -2.0, dtype=torch.float32, device=DEV)
    assert lib.nm_scale_search(Wd.data_ptr(), rows, cols, cols, N, M, bits, rps, C, s_ws.data_ptr(), ws.data_ptr(), need, st) == 0
    assert lib.nm_scale_search_static(Wd.data_ptr(), rows, cols, cols, N, M, bits, rps, C, s_st.data_ptr(), st) == 0
    torch.cuda.synchronize()
    return s_ws.cpu().numpy(), s_st.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one():
    lib = binding.raw()
    rng = np.random.default_rng(71)
    # the larger problem first (fills 3072 x 17 partial errors of the array), then a smaller one, then a third shape
    for rows, cols, N, M, bits, rps, C in [(3072, 768, 2, 4, 4, 32, 32), (70, 256, 2, 4, 4, 1, 32), (257, 512, 1, 4, 8, 5, 64)]:
        print("static scratch", rows, cols, N, M, bits, rps, C, flush=True)
        W = (rng.standard_normal((rows, cols)) * rng.random((rows, 1)) * 0.05).astype(np.float32)
        W[::5] *= np.linspace(0.05, 4.0, cols).astype(np.float32)
        W[3] = 0.0
        s_ws, s_st = both(lib, W, N, M, bits, rps, C)
        assert np.array_equal(s_ws.view(np.uint32), s_st.view(np.uint32)), "scales differ between the two entry points"
        assert np.all(s_st > 0)
        # and both are the oracle's scales (up to candidates whose errors tie to 1e-12, see the parity suite)
        s_ref, err = oracle.dist_scales(W, N, M, bits, rps, C)
        same = s_st == s_ref
        assert np.count_nonzero(~same) <= 0.02 * rows
    # beyond the array: refused, nothing enqueued (the pointers are never touched)
    P = 0x1000
    rows = (2 << 20) // (33 * 8) + 1
    assert lib.nm_scale_search_static(P, rows, 8, 8, 2, 4, 8, 1, 64, P, None) == -10
    assert lib.nm_scale_search_static(P, rows - 1, 8, 8, 2, 4, 8, 0, 64, P, None) == -2      # other checks as for nm_scale_search
