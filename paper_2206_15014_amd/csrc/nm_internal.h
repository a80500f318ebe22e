// Internal launch interfaces between the C-ABI front end (nm_api.hip) and the kernel files.
#ifndef NM_INTERNAL_H
#define NM_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>

#include <atomic>

namespace nm {

// ---------------------------------------------------------------------------------------------
// Where a byte of a packed array lives, in either layout of include/nm.h.  `ub` = bytes per
// unit (the packed bytes of one row that cover 32 input columns), `stride` = bytes per row in
// the row layout, `slices` = cols / 128.
// ---------------------------------------------------------------------------------------------
__host__ __device__ constexpr int piece_bytes(int ub)
{
    return (ub % 16 == 0) ? 16 : (ub % 8 == 0) ? 8 : (ub % 4 == 0) ? 4 : (ub % 2 == 0) ? 2 : 1;
}

__host__ __device__ inline size_t tiled_offset(uint32_t row, uint32_t byte_in_row, uint32_t ub, uint32_t slices)
{
    const uint32_t u = byte_in_row / ub, i = byte_in_row % ub;
    const uint32_t pb = (uint32_t)piece_bytes((int)ub);
    const size_t block = (size_t)(row >> 4) * slices + (u >> 2);
    return block * 64 * ub + ((i / pb) * 64 + (u & 3) * 16 + (row & 15)) * pb + i % pb;
}

struct PackedArray {
    int tiled;             // nm_layout
    uint32_t ub;           // bytes per unit (0: the array does not exist - metadata of a dense matrix)
    uint32_t stride;       // bytes per row, row layout
    uint32_t slices;       // cols / 128, tiled layout
    __host__ __device__ size_t at(uint32_t row, uint32_t byte_in_row) const
    {
        return tiled ? tiled_offset(row, byte_in_row, ub, slices) : (size_t)row * stride + byte_in_row;
    }
};

inline int index_bits(int N, int M) { return N >= M ? 0 : (M == 4 ? 2 : 4); }

inline PackedArray packed_values(int cols, int N, int M, int bits, int layout)
{
    const size_t kc = (size_t)cols / M * N;
    return PackedArray{layout, (uint32_t)(32 / M * N * bits / 8), (uint32_t)((kc * bits + 7) / 8), (uint32_t)(cols / 128)};
}
inline PackedArray packed_meta(int cols, int N, int M, int layout)
{
    const size_t kc = (size_t)cols / M * N;
    const int ib = index_bits(N, M);
    return PackedArray{layout, (uint32_t)(32 / M * N * ib / 8), (uint32_t)((kc * ib + 7) / 8), (uint32_t)(cols / 128)};
}
// bytes of the whole array for `rows` rows
inline size_t packed_bytes(const PackedArray& p, int rows, int cols)
{
    return p.tiled ? (size_t)((rows + 15) / 16) * 16 * (size_t)(cols / 32) * p.ub : (size_t)rows * p.stride;
}

struct GemmArgs {
    const int8_t* X;       // [tokens][ldx]
    int tokens, K, ldx;
    float act_scale;
    const float* act_scale_dev;   // replaces act_scale when given
    const uint8_t* vals;   // packed weights of an O x K matrix
    const uint8_t* meta;
    const float* scales;   // [O]
    int O, N, M, bits;
    PackedArray pv, pm;    // layout of vals / meta
    const float* bias;     // [O] or null
    int32_t* acc;          // [tokens][ldo] or null
    void* out;             // [tokens][ldo] or null
    int out_dtype;         // nm_out_dtype; 3 = int8 codes (nm_gemm_q8)
    int ldo;
    int store_through;     // set by a launcher: output stores bypass the L2's write-back (large outputs)
    int k_rotate;          // set by a launcher: workgroups start their walk along K at different blocks
    float out_scale;       // out_dtype 3: scale of the output codes
    const float* out_scale_dev;   // replaces out_scale when given
    float* absmax;         // out_dtype 3: max |y| is max-combined into it, or null
};

// Several GEMMs of one pattern in one launch (nm_gemm_batch): the items' tiles are numbered one
// item after the other.
constexpr int GEMM_BATCH_MAX = 4;
struct GemmBatch {
    GemmArgs item[GEMM_BATCH_MAX];
    int first_tile[GEMM_BATCH_MAX + 1];    // item i owns tiles [first_tile[i], first_tile[i + 1])
    int tiles_o[GEMM_BATCH_MAX];           // column tiles of item i
    int count;
};

// Launch-error bracket: begin_launch() drops any stale error left in this thread by earlier HIP
// calls of the caller; launch_status() reports what the launch itself produced.
inline void begin_launch() { (void)hipGetLastError(); }
inline int launch_status()
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return 0;
    fprintf(stderr, "libnm: kernel launch failed: %s\n", hipGetErrorString(e));
    return -7;
}

// Kernels whose LDS ring exceeds 64 KB need their dynamic-LDS limit raised, an attribute a device
// keeps per kernel: `done` (one word per kernel instantiation) has a bit per device that has it.
// Two threads may both raise it the first time; that is harmless.
inline void raise_lds_limit(const void* kernel, size_t lds_bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    done.fetch_or(bit, std::memory_order_release);
}

// Each returns 0 or NM_ERR_HIP (-7).
int launch_compress(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int layout, int rows_per_scale,
                    void* vals, void* meta, float* scales, hipStream_t st);
struct CompressItem {
    const float* W;
    int rows, cols, ldw;
    void* vals;
    void* meta;
    float* scales;
};
int launch_compress_batch(const CompressItem* items, int count, int N, int M, int bits, int layout, hipStream_t st);
void launch_group_scales(const float* W, int rows, int cols, int ldw, int rows_per_scale, float qmax, float* scales,
                         hipStream_t st);
int launch_repack(const void* vals_in, const void* meta_in, int rows, int cols, int N, int M, int bits, int layout_in,
                  void* vals_out, void* meta_out, hipStream_t st);
int launch_decompress(const void* vals, const void* meta, int rows, int cols, int N, int M, int bits, int layout,
                      int8_t* Wq, hipStream_t st);
int launch_project(const float* W, const float* U, int rows, int cols, int ldw, int N, int M, int bits,
                   int rows_per_scale, float* Z, float* U_out, int ldz, float* scales, hipStream_t st);
int launch_scale_search(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                        int candidates, float* scales, double* row_errors, hipStream_t st);
int launch_scale_search_static(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                               int candidates, float* scales, hipStream_t st);
int launch_absmax_to_scale(float* absmax, float* scale, int reset, hipStream_t st);
int launch_absmax_f32(const float* X, int tokens, int K, int ldx, float* absmax, hipStream_t st);
int launch_quantize_act(const float* X, int tokens, int K, int ldx, float scale, const float* scale_dev, int8_t* Q, int ldq,
                        hipStream_t st);
int launch_smfmac_probe(int blocks, int iters, unsigned long long* counters, hipStream_t st);
int launch_gemm(const GemmArgs& a, hipStream_t st);
// `count` (1 .. GEMM_BATCH_MAX) GEMMs of one pattern, layout and output type: one launch where the
// LDS-direct kernels cover every item, else one launch per item.
int launch_gemm_batch(const GemmArgs* items, int count, hipStream_t st);
// LDS-direct kernels (tiled layout), `count` items in one launch.  `cfg` 0 = the launcher's own
// tile choice, otherwise a forced variant; false: not handled, nothing launched.
bool launch_gemm_dma(const GemmArgs* items, int count, hipStream_t st, int cfg);

// Tile variant forced by the tests (0 = automatic), see nm_test_hooks.h.
int forced_gemm_tile();
// Records which kernel variant the last nm_gemm / nm_gemm_q8 / nm_gemm_batch call launched (the tile ids
// of the LDS-direct kernels, 1 .. 3 for the register-staged shapes, -1 for the one-thread-per-output
// kernel): read back by bench.py to group a step's launches by kernel.
void note_gemm_tile(int cfg);

}  // namespace nm

#endif
