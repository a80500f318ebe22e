// Internal launch interfaces between the C-ABI front end (nm_api.hip) and the kernel files.
#ifndef NM_INTERNAL_H
#define NM_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>

namespace nm {

struct GemmArgs {
    const int8_t* X;       // [tokens][ldx]
    int tokens, K, ldx;
    float act_scale;
    const uint8_t* vals;   // packed weights of an O x K matrix
    const uint8_t* meta;
    const float* scales;   // [O]
    int O, N, M, bits;
    const float* bias;     // [O] or null
    int32_t* acc;          // [tokens][ldo] or null
    void* out;             // [tokens][ldo] or null
    int out_dtype;         // nm_out_dtype; 3 = int8 codes (nm_gemm_q8)
    int ldo;
    int vstride, mstride;  // packed row strides in bytes
    int store_through;     // set by a launcher: output stores bypass the L2's write-back (large outputs)
    int k_rotate;          // set by a launcher: workgroups start their walk along K at different blocks
    float out_scale;       // out_dtype 3: scale of the output codes
    float* absmax;         // out_dtype 3: max |y| is max-combined into it, or null
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

// Each returns 0 or NM_ERR_HIP (-7).
int launch_compress(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                    void* vals, void* meta, float* scales, hipStream_t st);
struct CompressItem {
    const float* W;
    int rows, cols, ldw;
    void* vals;
    void* meta;
    float* scales;
};
int launch_compress_batch(const CompressItem* items, int count, int N, int M, int bits, hipStream_t st);
void launch_group_scales(const float* W, int rows, int cols, int ldw, int rows_per_scale, float qmax, float* scales,
                         hipStream_t st);
int launch_decompress(const void* vals, const void* meta, int rows, int cols, int N, int M, int bits,
                      int8_t* Wq, hipStream_t st);
int launch_project(const float* W, const float* U, int rows, int cols, int ldw, int N, int M, int bits,
                   int rows_per_scale, float* Z, float* U_out, int ldz, float* scales, hipStream_t st);
int launch_gemm(const GemmArgs& a, hipStream_t st);
bool launch_gemm_dma(const GemmArgs& a, hipStream_t st, int cfg);      // false: not handled, nothing launched
bool launch_gemm_stream(const GemmArgs& a, hipStream_t st, int cfg);   // same
bool launch_gemm_xres(const GemmArgs& a, hipStream_t st, int cfg);    // same

}  // namespace nm

#endif
