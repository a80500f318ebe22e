// C-ABI front end of libnm (declared in include/nm.h): host-side argument validation and dispatch.
// Nothing here touches the GPU before the arguments have been accepted.
#include <hip/hip_runtime.h>

#include <vector>

#include "nm.h"
#include "nm_internal.h"

namespace {

int check_pattern(int rows, int cols, int N, int M, int bits)
{
    if (rows <= 0 || cols <= 0) return NM_ERR_DIM;
    if (M != 4 && M != 8) return NM_ERR_PATTERN;
    if (N < 1 || N >= M) return NM_ERR_PATTERN;
    if (cols % M != 0) return NM_ERR_PATTERN;
    if (bits != 4 && bits != 8) return NM_ERR_BITS;
    return NM_OK;
}

size_t row_bytes(size_t entries, int bits_per_entry) { return (entries * bits_per_entry + 7) / 8; }

}  // namespace

extern "C" {

int nm_packed_sizes(int rows, int cols, int N, int M, int bits,
                    size_t* vals_bytes, size_t* meta_bytes, size_t* scales_bytes)
{
    const int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    const size_t kc = (size_t)cols / M * N;
    if (vals_bytes) *vals_bytes = (size_t)rows * row_bytes(kc, bits);
    if (meta_bytes) *meta_bytes = (size_t)rows * row_bytes(kc, M == 4 ? 2 : 4);
    if (scales_bytes) *scales_bytes = (size_t)rows * sizeof(float);
    return NM_OK;
}

int nm_compress(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits,
                void* vals_dev, void* meta_dev, float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!W_dev || !vals_dev || !meta_dev || !scales_dev) return NM_ERR_NULL;
    if (ldw < cols) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4) return NM_ERR_ALIGN;
    return nm::launch_compress(W_dev, rows, cols, ldw, N, M, bits, 1, vals_dev, meta_dev, scales_dev,
                               static_cast<hipStream_t>(hip_stream));
}

int nm_compress_grouped(const float* W_dev, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                        void* vals_dev, void* meta_dev, float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!W_dev || !vals_dev || !meta_dev || !scales_dev) return NM_ERR_NULL;
    if (ldw < cols || rows_per_scale < 1) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 4 || (uintptr_t)scales_dev % 4) return NM_ERR_ALIGN;
    return nm::launch_compress(W_dev, rows, cols, ldw, N, M, bits, rows_per_scale, vals_dev, meta_dev, scales_dev,
                               static_cast<hipStream_t>(hip_stream));
}

int nm_compress_batch(const nm_compress_item* items, int count, int N, int M, int bits, void* hip_stream)
{
    if (count <= 0 || count > NM_COMPRESS_BATCH_MAX_ITEMS) return NM_ERR_DIM;
    if (!items) return NM_ERR_NULL;
    std::vector<nm::CompressItem> v((size_t)count);
    for (int i = 0; i < count; ++i) {
        const nm_compress_item& c = items[i];
        const int rc = check_pattern(c.rows, c.cols, N, M, bits);
        if (rc) return rc;
        if (!c.W_dev || !c.vals_dev || !c.meta_dev || !c.scales_dev) return NM_ERR_NULL;
        if (c.ldw < c.cols) return NM_ERR_DIM;
        if ((uintptr_t)c.W_dev % 4 || (uintptr_t)c.scales_dev % 4) return NM_ERR_ALIGN;
        v[(size_t)i] = nm::CompressItem{c.W_dev, c.rows, c.cols, c.ldw, c.vals_dev, c.meta_dev, c.scales_dev};
    }
    return nm::launch_compress_batch(v.data(), count, N, M, bits, static_cast<hipStream_t>(hip_stream));
}

int nm_decompress_i8(const void* vals_dev, const void* meta_dev, int rows, int cols,
                     int N, int M, int bits, int8_t* Wq_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits);
    if (rc) return rc;
    if (!vals_dev || !meta_dev || !Wq_dev) return NM_ERR_NULL;
    return nm::launch_decompress(vals_dev, meta_dev, rows, cols, N, M, bits, Wq_dev,
                                 static_cast<hipStream_t>(hip_stream));
}

int nm_gemm(const int8_t* X_dev, int tokens, int K, int ldx, float act_scale,
            const void* vals_dev, const void* meta_dev, const float* scales_dev,
            int O, int N, int M, int bits,
            const float* bias_dev, int32_t* acc_dev, void* out_dev, int out_dtype,
            int ldo, void* hip_stream)
{
    const int rc = check_pattern(O, K, N, M, bits);
    if (rc) return rc;
    if (tokens <= 0) return NM_ERR_DIM;
    if (!X_dev || !vals_dev || !meta_dev || !scales_dev) return NM_ERR_NULL;
    if (out_dtype != NM_OUT_NONE && out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
    if ((out_dtype == NM_OUT_NONE) != (out_dev == nullptr)) return NM_ERR_DTYPE;
    if (!acc_dev && !out_dev) return NM_ERR_NULL;
    if (ldx < K || ldo < O) return NM_ERR_DIM;
    if ((uintptr_t)scales_dev % 4 || (uintptr_t)bias_dev % 4 || (uintptr_t)acc_dev % 4 ||
        (uintptr_t)out_dev % (out_dtype == NM_OUT_BF16 ? 2 : 4))
        return NM_ERR_ALIGN;

    nm::GemmArgs a;
    a.X = X_dev; a.tokens = tokens; a.K = K; a.ldx = ldx; a.act_scale = act_scale;
    a.vals = static_cast<const uint8_t*>(vals_dev);
    a.meta = static_cast<const uint8_t*>(meta_dev);
    a.scales = scales_dev;
    a.O = O; a.N = N; a.M = M; a.bits = bits;
    a.bias = bias_dev; a.acc = acc_dev; a.out = out_dev; a.out_dtype = out_dtype; a.ldo = ldo;
    const size_t kc = (size_t)K / M * N;
    a.vstride = (int)row_bytes(kc, bits);
    a.mstride = (int)row_bytes(kc, M == 4 ? 2 : 4);
    a.store_through = 0;
    a.k_rotate = 0;
    a.out_scale = 1.0f;
    a.absmax = nullptr;
    return nm::launch_gemm(a, static_cast<hipStream_t>(hip_stream));
}

int nm_project(const float* W_dev, const float* U_dev, int rows, int cols, int ldw,
               int N, int M, int bits, int rows_per_scale,
               float* Z_dev, float* U_out_dev, int ldz, float* scales_dev, void* hip_stream)
{
    const int rc = check_pattern(rows, cols, N, M, bits ? bits : 8);
    if (rc) return rc;
    if (!W_dev || !Z_dev || (bits && !scales_dev)) return NM_ERR_NULL;
    if (ldw < cols || ldz < cols || rows_per_scale < 1) return NM_ERR_DIM;
    if ((uintptr_t)W_dev % 16 || (uintptr_t)U_dev % 16 || (uintptr_t)Z_dev % 16 || (uintptr_t)U_out_dev % 16 ||
        (uintptr_t)scales_dev % 4 || ldw % 4 || ldz % 4)
        return NM_ERR_ALIGN;
    return nm::launch_project(W_dev, U_dev, rows, cols, ldw, N, M, bits, rows_per_scale, Z_dev, U_out_dev, ldz,
                              scales_dev, static_cast<hipStream_t>(hip_stream));
}

int nm_gemm_q8(const int8_t* X_dev, int tokens, int K, int ldx, float act_scale,
               const void* vals_dev, const void* meta_dev, const float* scales_dev,
               int O, int N, int M, int bits,
               const float* bias_dev, float out_scale,
               int8_t* out_dev, int ldo, float* absmax_dev, void* hip_stream)
{
    const int rc = check_pattern(O, K, N, M, bits);
    if (rc) return rc;
    if (tokens <= 0) return NM_ERR_DIM;
    if (!X_dev || !vals_dev || !meta_dev || !scales_dev || !out_dev) return NM_ERR_NULL;
    if (ldx < K || ldo < O) return NM_ERR_DIM;
    if (!(out_scale > 0.0f) || !(out_scale <= 3.402823466e38f)) return NM_ERR_DIM;
    if ((uintptr_t)scales_dev % 4 || (uintptr_t)bias_dev % 4 || (uintptr_t)absmax_dev % 4 || (uintptr_t)out_dev % 4)
        return NM_ERR_ALIGN;

    nm::GemmArgs a;
    a.X = X_dev; a.tokens = tokens; a.K = K; a.ldx = ldx; a.act_scale = act_scale;
    a.vals = static_cast<const uint8_t*>(vals_dev);
    a.meta = static_cast<const uint8_t*>(meta_dev);
    a.scales = scales_dev;
    a.O = O; a.N = N; a.M = M; a.bits = bits;
    a.bias = bias_dev; a.acc = nullptr; a.out = out_dev; a.out_dtype = 3; a.ldo = ldo;
    const size_t kc = (size_t)K / M * N;
    a.vstride = (int)row_bytes(kc, bits);
    a.mstride = (int)row_bytes(kc, M == 4 ? 2 : 4);
    a.store_through = 0;
    a.k_rotate = 0;
    a.out_scale = out_scale;
    a.absmax = absmax_dev;
    return nm::launch_gemm(a, static_cast<hipStream_t>(hip_stream));
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
        default: return "unknown status";
    }
}

}  // extern "C"
