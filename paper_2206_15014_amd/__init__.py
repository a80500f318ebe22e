"""N:M-sparse low-bit integer linear layers for MI355X (gfx950).

``nm_compress`` / ``nm_gemm`` and friends are thin marshalling wrappers over the
C-ABI library built from ``csrc/``; every step of the path runs in its HIP
kernels.  ``synth`` holds the seeded input generators and workload tables.
"""
from .binding import (  # noqa: F401
    NM_LAYOUT_ROWS,
    NM_LAYOUT_TILED,
    NMError,
    library_path,
    nm_absmax_f32,
    nm_absmax_to_scale,
    nm_compress,
    nm_compress_batch,
    nm_compress_grouped,
    nm_compress_scaled,
    nm_decompress_i8,
    nm_gemm,
    nm_gemm_batch,
    nm_gemm_q8,
    nm_packed_sizes,
    nm_project,
    nm_quantize_act,
    nm_repack,
    nm_scale_search,
    nm_scale_search_static,
    nm_status_string,
)
