// C-ABI front end of libnm (declared in include/nm.h): host-side argument validation and dispatch.
// Nothing here touches the GPU before the arguments have been accepted.
#include <hip/hip_runtime.h>

#include <atomic>
#include <vector>

#include "nm.h"
#include "nm_internal.h"
#include "nm_test_hooks.h"

namespace {

int check_pattern(int rows, int cols, int N, int M, int bits, int layout)
{
    if (rows <= 0 || cols <= 0) return NM_ERR_DIM;
    if (M != 4 && M != 8) return NM_ERR_PATTERN;
    if (N < 1 || N > M) return NM_ERR_PATTERN;
    if (cols % M != 0) return NM_ERR_PATTERN;
    if (bits != 4 && bits != 8) return NM_ERR_BITS;
    if (layout != NM_LAYOUT_ROWS && layout != NM_LAYOUT_TILED) return NM_ERR_LAYOUT;
    if (layout == NM_LAYOUT_TILED && cols % 128 != 0) return NM_ERR_PATTERN;
    return NM_OK;
}

// A dense matrix has one format whatever the group width it was declared with: the kernels see 4:4.
void canonical_dense(int& N, int& M)
{
    if (N == M) N = M = 4;
}

std::atomic<int> g_forced_tile{0};
std::atomic<int> g_last_tile{0};

}  // namespace

namespace nm {
int forced_gemm_tile() { return g_forced_tile.load(std::memory_order_relaxed); }
void note_gemm_tile(int cfg) { g_last_tile.store(cfg, std::memory_order_relaxed); }
}

extern "C" {

int nm_test_force_gemm_tile(int cfg) { return g_forced_tile.exchange(cfg, std::memory_order_relaxed); }

int nm_bench_last_gemm_tile(void) { return g_last_tile.load(std::memory_order_relaxed); }

int nm_bench_smfmac_probe(int blocks, int iters, unsigned long long* counters_dev, void* hip_stream)
{
    if (!counters_dev) return NM_ERR_NULL;
    if (blocks <= 0 || iters <= 0) return NM_ERR_DIM;
    return nm::launch_smfmac_probe(blocks, iters, counters_dev, static_cast<hipStream_t>(hip_stream));
}

int nm_packed_sizes(int rows, int cols, int N, int M, int bits, int layout,
                    size_t* vals_bytes, size_t* meta_bytes, size_t* scales_bytes)
{
    const int rc = check_pattern(rows, cols, N, M, bits, layout);
    if (rc) return rc;
    if (vals_bytes) *vals_bytes = nm::packed_bytes(nm::packed_values(cols, N, M, bits, layout), rows, cols);
    if (meta_bytes) *meta_bytes = nm::packed_bytes(nm::packed_meta(cols, N, M, layout), rows, cols);
    if (scales_bytes) *scales_bytes = (size_t)rows * sizeof(float);
    return NM_OK;
}

int nm_compress(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int layout,
                void* vals_dev, void* meta_dev, float* scales_dev, void* hip_stream)
{
    return nm_compress_grouped(W_dev, rows, cols, ldw, N, M, bits, layout, 1, vals_dev, meta_dev, scales_dev, hip_stream);
}

int nm_compress_grouped(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int layout, int rows_per_scale,
                        void* vals_dev, void* meta_dev, float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits, layout);
    if (rc) return rc;
    if (!W_dev || !vals_dev || (!meta_dev && N < M) || !scales_dev) return NM_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4) return NM_ERR_ALIGN;
    canonical_dense(N, M);
    return nm::launch_compress(W_dev, rows, cols, ldw, N, M, bits, layout, rows_per_scale, vals_dev, meta_dev, scales_dev,
                               static_cast<hipStream_t>(hip_stream));
}

int nm_compress_scaled(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int layout,
                       const float* scales_dev, void* vals_dev, void* meta_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits, layout);
    if (rc) return rc;
    if (!W_dev || !vals_dev || (!meta_dev && N < M) || !scales_dev) return NM_ERR_NULL;
    if (ldw < cols) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4) return NM_ERR_ALIGN;
    canonical_dense(N, M);
    // rows_per_scale 0: the kernels quantise with the scales they find (and leave the array as it is)
    return nm::launch_compress(W_dev, rows, cols, ldw, N, M, bits, layout, 0, vals_dev, meta_dev, const_cast<float*>(scales_dev),
                               static_cast<hipStream_t>(hip_stream));
}

size_t nm_scale_search_workspace_bytes(int rows, int candidates)
{
    if (rows <= 0 || candidates < 2 || candidates > 64 || candidates % 2) return 0;
    return (size_t)rows * (size_t)(candidates / 2 + 1) * sizeof(double);
}

int nm_scale_search(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale, int candidates,
                    float* scales_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits, NM_LAYOUT_ROWS);
    if (rc) return rc;
    if (!W_dev || !scales_dev || !workspace_dev) return NM_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1 || candidates < 2 || candidates > 64 || candidates % 2) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4 || (uintptr_t)workspace_dev % 8) return NM_ERR_ALIGN;
    if (workspace_bytes < nm_scale_search_workspace_bytes(rows, candidates)) return NM_ERR_WORKSPACE;
    return nm::launch_scale_search(W_dev, rows, cols, ldw, N, M, bits, rows_per_scale, candidates, scales_dev,
                                   static_cast<double*>(workspace_dev), static_cast<hipStream_t>(hip_stream));
}

int nm_scale_search_static(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale, int candidates,
                           float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits, NM_LAYOUT_ROWS);
    if (rc) return rc;
    if (!W_dev || !scales_dev) return NM_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1 || candidates < 2 || candidates > 64 || candidates % 2) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4) return NM_ERR_ALIGN;
    const size_t need = nm_scale_search_workspace_bytes(rows, candidates);
    if (need > NM_SCALE_SEARCH_STATIC_MAX_BYTES) {
        fprintf(stderr, "libnm: nm_scale_search_static: %d rows x %d candidates need %zu bytes of scratch, the built-in array holds %zu; "
                        "use nm_scale_search with a workspace\n", rows, candidates / 2 + 1, need, (size_t)NM_SCALE_SEARCH_STATIC_MAX_BYTES);
        return NM_ERR_WORKSPACE;
    }
    return nm::launch_scale_search_static(W_dev, rows, cols, ldw, N, M, bits, rows_per_scale, candidates, scales_dev,
                                          static_cast<hipStream_t>(hip_stream));
}

int nm_compress_batch(const nm_compress_item* items, int count, int N, int M, int bits, int layout, void* hip_stream)
{
    if (count <= 0 || count > NM_COMPRESS_BATCH_MAX_ITEMS) return NM_ERR_DIM;
    if (!items) return NM_ERR_NULL;
    std::vector<nm::CompressItem> v((size_t)count);
    for (int i = 0; i < count; ++i) {
        const nm_compress_item& c = items[i];
        const int rc = check_pattern(c.rows, c.cols, N, M, bits, layout);
        if (rc) return rc;
        if (!c.W_dev || !c.vals_dev || (!c.meta_dev && N < M) || !c.scales_dev) return NM_ERR_NULL;
        if (c.ldw < c.cols) return NM_ERR_DIM;
        if ((uintptr_t)c.W_dev % 4 || (uintptr_t)c.scales_dev % 4) return NM_ERR_ALIGN;
        v[(size_t)i] = nm::CompressItem{c.W_dev, c.rows, c.cols, c.ldw, c.vals_dev, c.meta_dev, c.scales_dev};
    }
    canonical_dense(N, M);
    return nm::launch_compress_batch(v.data(), count, N, M, bits, layout, static_cast<hipStream_t>(hip_stream));
}

int nm_repack(const void* vals_in_dev, const void* meta_in_dev, int rows, int cols, int N, int M, int bits, int layout_in,
              void* vals_out_dev, void* meta_out_dev, void* hip_stream)
{
    int rc = check_pattern(rows, cols, N, M, bits, layout_in);
    if (rc) return rc;
    rc = check_pattern(rows, cols, N, M, bits, NM_LAYOUT_TILED);     // the other side is tiled, or this one is
    if (rc) return rc;
    if (!vals_in_dev || !vals_out_dev || ((!meta_in_dev || !meta_out_dev) && N < M)) return NM_ERR_NULL;
    return nm::launch_repack(vals_in_dev, meta_in_dev, rows, cols, N, M, bits, layout_in, vals_out_dev, meta_out_dev,
                             static_cast<hipStream_t>(hip_stream));
}

int nm_decompress_i8(const void* vals_dev, const void* meta_dev, int rows, int cols,
                     int N, int M, int bits, int layout, int8_t* Wq_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits, layout);
    if (rc) return rc;
    if (!vals_dev || (!meta_dev && N < M) || !Wq_dev) return NM_ERR_NULL;
    canonical_dense(N, M);
    return nm::launch_decompress(vals_dev, meta_dev, rows, cols, N, M, bits, layout, Wq_dev,
                                 static_cast<hipStream_t>(hip_stream));
}

namespace {

// Validation common to nm_gemm and nm_gemm_q8, and the argument block of the launchers.
int gemm_args(nm::GemmArgs& a, const int8_t* X_dev, int tokens, int K, int ldx, float act_scale, const float* act_scale_dev,
              const void* vals_dev, const void* meta_dev, const float* scales_dev, int O, int N, int M, int bits, int layout,
              const float* bias_dev, int ldo)
{
    const int rc = check_pattern(O, K, N, M, bits, layout);
    if (rc) return rc;
    if (tokens <= 0) return NM_ERR_DIM;
    if (!X_dev || !vals_dev || (!meta_dev && N < M) || !scales_dev) return NM_ERR_NULL;
    if (ldx < K || ldo < O) return NM_ERR_DIM;
    if ((uintptr_t)scales_dev % 4 || (uintptr_t)bias_dev % 4 || (uintptr_t)act_scale_dev % 4) return NM_ERR_ALIGN;
    canonical_dense(N, M);
    a.X = X_dev; a.tokens = tokens; a.K = K; a.ldx = ldx; a.act_scale = act_scale; a.act_scale_dev = act_scale_dev;
    a.vals = static_cast<const uint8_t*>(vals_dev);
    a.meta = static_cast<const uint8_t*>(meta_dev);
    a.scales = scales_dev;
    a.O = O; a.N = N; a.M = M; a.bits = bits;
    a.pv = nm::packed_values(K, N, M, bits, layout);
    a.pm = nm::packed_meta(K, N, M, layout);
    a.bias = bias_dev; a.ldo = ldo;
    a.store_through = 0;
    a.k_rotate = 0;
    a.out_scale = 1.0f;
    a.out_scale_dev = nullptr;
    a.absmax = nullptr;
    return NM_OK;
}

}  // namespace

int nm_gemm(const int8_t* X_dev, int tokens, int K, int ldx, float act_scale, const float* act_scale_dev,
            const void* vals_dev, const void* meta_dev, const float* scales_dev,
            int O, int N, int M, int bits, int layout,
            const float* bias_dev, int32_t* acc_dev, void* out_dev, int out_dtype,
            int ldo, void* hip_stream)
{
    nm::GemmArgs a;
    const int rc = gemm_args(a, X_dev, tokens, K, ldx, act_scale, act_scale_dev, vals_dev, meta_dev, scales_dev, O, N, M, bits,
                             layout, bias_dev, ldo);
    if (rc) return rc;
    if (out_dtype != NM_OUT_NONE && out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
    if ((out_dtype == NM_OUT_NONE) != (out_dev == nullptr)) return NM_ERR_DTYPE;
    if (!acc_dev && !out_dev) return NM_ERR_NULL;
    if ((uintptr_t)acc_dev % 4 || (uintptr_t)out_dev % (out_dtype == NM_OUT_BF16 ? 2 : 4)) return NM_ERR_ALIGN;
    a.acc = acc_dev; a.out = out_dev; a.out_dtype = out_dtype;
    return nm::launch_gemm(a, static_cast<hipStream_t>(hip_stream));
}

int nm_gemm_batch(const nm_gemm_item* items, int count, int N, int M, int bits, int layout, int out_dtype, void* hip_stream)
{
    if (!items) return NM_ERR_NULL;
    if (count <= 0 || count > NM_GEMM_BATCH_MAX_ITEMS) return NM_ERR_DIM;
    static_assert(NM_GEMM_BATCH_MAX_ITEMS == nm::GEMM_BATCH_MAX, "the ABI's limit is the kernels' limit");
    if (out_dtype != NM_OUT_NONE && out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
    nm::GemmArgs a[NM_GEMM_BATCH_MAX_ITEMS];
    for (int i = 0; i < count; ++i) {
        const nm_gemm_item& it = items[i];
        const int rc = gemm_args(a[i], it.X_dev, it.tokens, it.K, it.ldx, it.act_scale, it.act_scale_dev, it.vals_dev, it.meta_dev,
                                 it.scales_dev, it.O, N, M, bits, layout, it.bias_dev, it.ldo);
        if (rc) return rc;
        if ((out_dtype == NM_OUT_NONE) != (it.out_dev == nullptr)) return NM_ERR_DTYPE;
        if (!it.acc_dev && !it.out_dev) return NM_ERR_NULL;
        if ((uintptr_t)it.acc_dev % 4 || (uintptr_t)it.out_dev % (out_dtype == NM_OUT_BF16 ? 2 : 4)) return NM_ERR_ALIGN;
        a[i].acc = it.acc_dev; a[i].out = it.out_dev; a[i].out_dtype = out_dtype;
    }
    return nm::launch_gemm_batch(a, count, static_cast<hipStream_t>(hip_stream));
}

int nm_project(const float* W_dev, const float* U_dev, int rows, int cols, int ldw,
               int N, int M, int bits, int rows_per_scale,
               float* Z_dev, float* U_out_dev, int ldz, float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits ? bits : 8, NM_LAYOUT_ROWS);
    if (rc) return rc;
    if (!W_dev || !Z_dev || (bits && !scales_dev)) return NM_ERR_NULL;
    if (ldw < cols || ldz < cols || rows_per_scale < 1) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 16 || (uintptr_t)U_dev % 16 || (uintptr_t)Z_dev % 16 || (uintptr_t)U_out_dev % 16 ||
        (uintptr_t)scales_dev % 4 || ldw % 4 || ldz % 4)
        return NM_ERR_ALIGN;
    return nm::launch_project(W_dev, U_dev, rows, cols, ldw, N, M, bits, rows_per_scale, Z_dev, U_out_dev, ldz,
                              scales_dev, static_cast<hipStream_t>(hip_stream));
}

int nm_gemm_q8(const int8_t* X_dev, int tokens, int K, int ldx, float act_scale, const float* act_scale_dev,
               const void* vals_dev, const void* meta_dev, const float* scales_dev,
               int O, int N, int M, int bits, int layout,
               const float* bias_dev, float out_scale, const float* out_scale_dev,
               int8_t* out_dev, int ldo, float* absmax_dev, void* hip_stream)
{
    nm::GemmArgs a;
    const int rc = gemm_args(a, X_dev, tokens, K, ldx, act_scale, act_scale_dev, vals_dev, meta_dev, scales_dev, O, N, M, bits,
                             layout, bias_dev, ldo);
    if (rc) return rc;
    if (!out_dev) return NM_ERR_NULL;
    if (!out_scale_dev && (!(out_scale > 0.0f) || !(out_scale <= 3.402823466e38f))) return NM_ERR_SCALE;
    if ((uintptr_t)absmax_dev % 4 || (uintptr_t)out_dev % 4 || (uintptr_t)out_scale_dev % 4) return NM_ERR_ALIGN;
    a.acc = nullptr; a.out = out_dev; a.out_dtype = 3;
    a.out_scale = out_scale;
    a.out_scale_dev = out_scale_dev;
    a.absmax = absmax_dev;
    return nm::launch_gemm(a, static_cast<hipStream_t>(hip_stream));
}

int nm_absmax_to_scale(float* absmax_dev, float* scale_dev, int reset, void* hip_stream)
{
    if (!absmax_dev || !scale_dev) return NM_ERR_NULL;
    if ((uintptr_t)absmax_dev % 4 || (uintptr_t)scale_dev % 4) return NM_ERR_ALIGN;
    if (absmax_dev == scale_dev) return NM_ERR_DIM;
    return nm::launch_absmax_to_scale(absmax_dev, scale_dev, reset, static_cast<hipStream_t>(hip_stream));
}

int nm_absmax_f32(const float* X_dev, int tokens, int K, int ldx, float* absmax_dev, void* hip_stream)
{
    if (!X_dev || !absmax_dev) return NM_ERR_NULL;
    if (tokens <= 0 || K <= 0 || ldx < K) return NM_ERR_DIM;
    if ((uintptr_t)X_dev % 4 || (uintptr_t)absmax_dev % 4) return NM_ERR_ALIGN;
    return nm::launch_absmax_f32(X_dev, tokens, K, ldx, absmax_dev, static_cast<hipStream_t>(hip_stream));
}

int nm_quantize_act(const float* X_dev, int tokens, int K, int ldx, float scale, const float* scale_dev,
                    int8_t* Xq_dev, int ldq, void* hip_stream)
{
    if (!X_dev || !Xq_dev) return NM_ERR_NULL;
    if (tokens <= 0 || K <= 0 || ldx < K || ldq < K) return NM_ERR_DIM;
    if (!scale_dev && (!(scale > 0.0f) || !(scale <= 3.402823466e38f))) return NM_ERR_SCALE;
    if ((uintptr_t)X_dev % 4 || (uintptr_t)scale_dev % 4) return NM_ERR_ALIGN;
    return nm::launch_quantize_act(X_dev, tokens, K, ldx, scale, scale_dev, Xq_dev, ldq, static_cast<hipStream_t>(hip_stream));
}

const char* nm_status_string(int status)
{
    switch (status) {
        case NM_OK: return "ok";
        case NM_ERR_NULL: return "required pointer is null";
        case NM_ERR_DIM: return "bad dimension or leading dimension";
        case NM_ERR_PATTERN: return "unsupported N:M pattern for this width";
        case NM_ERR_BITS: return "weight bits must be 4 or 8";
        case NM_ERR_DTYPE: return "bad output dtype / output pointer combination";
        case NM_ERR_ALIGN: return "pointer or leading dimension misaligned";
        case NM_ERR_HIP: return "HIP launch error";
        case NM_ERR_LAYOUT: return "unknown layout of the packed buffers";
        case NM_ERR_SCALE: return "scale is not a positive finite number";
        case NM_ERR_WORKSPACE: return "workspace smaller than the size query says";
        default: return "unknown status";
    }
}

}  // extern "C"
