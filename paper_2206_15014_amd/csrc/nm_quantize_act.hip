// nm_absmax_f32 / nm_quantize_act kernels for gfx950.
//
// A floating-point activation tensor as the 8-bit integers the layers take (Sec. 5.3): one
// scale for the whole tensor from its largest magnitude (the rule of Sec. 3.3.1 at 8 bits),
// then the symmetric quantiser of Sec. 3.3 (Eq. 5, offset 0) per element.  Two passes over
// the tensor, each bound by HBM: the first reads 4 bytes per element, the second reads 4 and
// writes 1.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "nm_quantize.h"

namespace nm {

namespace {

typedef float v4f_t __attribute__((ext_vector_type(4)));

constexpr int ACT_THREADS = 256;
constexpr int ACT_VECS = 4;          // 16-byte pieces per thread, one block-width apart
constexpr int ACT_MAX_ROWS = 65535;  // grid.y limit; further rows by a stride loop

// max over the 64 lanes of a non-negative value, valid in lane 63: each step adds the lanes
// 1, 2, 4, 8 below inside a row of 16, then the rows are chained by the two row broadcasts.
__device__ __forceinline__ float wave_max_last_lane(float m)
{
    // a lane without a source in a step receives 0, the identity for non-negative values
#define NM_MAX_STEP(ctrl, row_mask) \
    m = fmaxf(m, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(m), ctrl, row_mask, 0xF, false)))
    NM_MAX_STEP(0x111, 0xF);   // row_shr:1
    NM_MAX_STEP(0x112, 0xF);   // row_shr:2
    NM_MAX_STEP(0x114, 0xF);   // row_shr:4
    NM_MAX_STEP(0x118, 0xF);   // row_shr:8
    NM_MAX_STEP(0x142, 0xA);   // row_bcast:15 -> rows 1 and 3
    NM_MAX_STEP(0x143, 0xC);   // row_bcast:31 -> rows 2 and 3
#undef NM_MAX_STEP
    return m;
}

// The statistic is one word for the whole chip, and atomics on one address are served one after
// the other by the memory side (about 10 ns each): one per wavefront of a 25 MB tensor would take
// ten times longer than reading it.  So the reduction runs in few, large workgroups that stride
// over the tensor - at most one per compute unit - and each commits once.
constexpr int MAX_THREADS = 1024;
constexpr int MAX_BLOCKS = 256;
constexpr int MAX_UNROLL = 4;        // loads in flight per lane

// Non-negative floats order like their bit patterns, so the running maximum is an unsigned max.
// Every thread of the workgroup must call it.
__device__ __forceinline__ void commit_max(float* absmax, float m)
{
    __shared__ float part[MAX_THREADS / 64];
    m = wave_max_last_lane(m);
    if ((threadIdx.x & 63) == 63) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < MAX_THREADS / 64; ++w) m = fmaxf(m, part[w]);
        unsigned int* u = reinterpret_cast<unsigned int*>(absmax);      // often a larger value is already there
        if (__float_as_uint(m) > __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(u, __float_as_uint(m));
    }
}

// Rows of whole 16-byte pieces: `vecs` pieces per row, rows `ldx4` pieces apart; DENSE: one row.
template <bool DENSE>
__global__ __launch_bounds__(MAX_THREADS) void absmax_vec_kernel(const v4f_t* __restrict__ X, long long total, long long vecs,
                                                                 long long ldx4, float* absmax)
{
    float m = 0.0f;
    const long long sweep = (long long)gridDim.x * MAX_THREADS;
    for (long long v0 = (long long)blockIdx.x * MAX_THREADS + threadIdx.x; v0 < total; v0 += MAX_UNROLL * sweep) {
        v4f_t x[MAX_UNROLL];
#pragma unroll
        for (int i = 0; i < MAX_UNROLL; ++i) {
            const long long v = v0 + i * sweep;
            x[i] = v4f_t{0.0f, 0.0f, 0.0f, 0.0f};
            if (v < total) {
                long long at = v;
                if constexpr (!DENSE) {
                    const long long t = v / vecs;
                    at = t * ldx4 + (v - t * vecs);
                }
                x[i] = __builtin_nontemporal_load(X + at);
            }
        }
#pragma unroll
        for (int i = 0; i < MAX_UNROLL; ++i)
            m = fmaxf(fmaxf(m, fmaxf(fabsf(x[i].x), fabsf(x[i].y))), fmaxf(fabsf(x[i].z), fabsf(x[i].w)));
    }
    commit_max(absmax, m);
}

// Any shape and alignment: one element per lane and step.
__global__ __launch_bounds__(MAX_THREADS) void absmax_any_kernel(const float* __restrict__ X, long long total, long long K,
                                                                 long long ldx, float* absmax)
{
    float m = 0.0f;
    const long long sweep = (long long)gridDim.x * MAX_THREADS;
    for (long long e = (long long)blockIdx.x * MAX_THREADS + threadIdx.x; e < total; e += sweep) {
        const long long t = e / K;
        m = fmaxf(m, fabsf(X[t * ldx + (e - t * K)]));
    }
    commit_max(absmax, m);
}

// Eq. 5 at 8 bits on one element.  |x| beyond 128 s is brought to 128 s first (an exact product
// for the scales the reciprocal route takes): its code is the clamp's +-127 either way, and the
// quotient's intermediates then stay far from overflow whatever the caller's scale is.
template <bool RECIP>
__device__ __forceinline__ int act_code(float x, const Divisor<RECIP>& d, float bound)
{
    if constexpr (RECIP) x = fminf(fmaxf(x, -bound), bound);
    return quantize<8>(x, d);
}

template <bool RECIP>
__device__ __forceinline__ void quantize_vec_rows(const v4f_t* __restrict__ X, int tokens, long long vecs, long long ldx4,
                                                  uint32_t* __restrict__ Q, long long ldq4, const Divisor<RECIP> d)
{
    const float bound = d.s * 128.0f;
    const long long v0 = (long long)blockIdx.x * (ACT_THREADS * ACT_VECS) + threadIdx.x;
    for (int t = blockIdx.y; t < tokens; t += gridDim.y) {
        const v4f_t* row = X + (long long)t * ldx4;
        uint32_t* out = Q + (long long)t * ldq4;
        v4f_t x[ACT_VECS];
#pragma unroll
        for (int i = 0; i < ACT_VECS; ++i) {
            const long long v = v0 + (long long)i * ACT_THREADS;
            if (v < vecs) x[i] = __builtin_nontemporal_load(row + v);
        }
#pragma unroll
        for (int i = 0; i < ACT_VECS; ++i) {
            const long long v = v0 + (long long)i * ACT_THREADS;
            if (v < vecs) {
                const uint32_t c = ((uint32_t)act_code(x[i].x, d, bound) & 0xFFu) | (((uint32_t)act_code(x[i].y, d, bound) & 0xFFu) << 8) |
                                   (((uint32_t)act_code(x[i].z, d, bound) & 0xFFu) << 16) | ((uint32_t)act_code(x[i].w, d, bound) << 24);
                out[v] = c;
            }
        }
    }
}

// The scale is one value for the whole launch, so the choice of division route is uniform.
__device__ __forceinline__ bool reciprocal_route(float s) { return s >= 0x1p-60f && s <= 0x1p60f; }

__global__ __launch_bounds__(ACT_THREADS) void quantize_act_vec_kernel(const v4f_t* __restrict__ X, int tokens, long long vecs,
                                                                       long long ldx4, float scale, const float* scale_dev,
                                                                       uint32_t* __restrict__ Q, long long ldq4)
{
    const float s = scale_dev ? *scale_dev : scale;
    if (reciprocal_route(s)) quantize_vec_rows(X, tokens, vecs, ldx4, Q, ldq4, Divisor<true>{s, __fdiv_rn(1.0f, s)});
    else quantize_vec_rows(X, tokens, vecs, ldx4, Q, ldq4, Divisor<false>{s, 0.0f});
}

__global__ __launch_bounds__(ACT_THREADS) void quantize_act_any_kernel(const float* __restrict__ X, int tokens, int K, long long ldx,
                                                                       float scale, const float* scale_dev, int8_t* __restrict__ Q,
                                                                       long long ldq)
{
    const float s = scale_dev ? *scale_dev : scale;
    const long long k = (long long)blockIdx.x * ACT_THREADS + threadIdx.x;
    if (k >= K) return;
    const Divisor<false> d{s, 0.0f};
    for (int t = blockIdx.y; t < tokens; t += gridDim.y)
        Q[(long long)t * ldq + k] = (int8_t)quantize<8>(X[(long long)t * ldx + k], d);
}

// A tensor whose rows follow each other without padding is one long row.
struct Rows {
    int tokens;
    long long K;
};
Rows flatten(int tokens, int K, bool dense)
{
    return dense ? Rows{1, (long long)tokens * K} : Rows{tokens, (long long)K};
}

dim3 vec_grid(const Rows& r)
{
    const long long per_block = (long long)ACT_THREADS * ACT_VECS * 4;
    return dim3((unsigned)((r.K + per_block - 1) / per_block), (unsigned)(r.tokens < ACT_MAX_ROWS ? r.tokens : ACT_MAX_ROWS));
}

dim3 any_grid(int tokens, int K)
{
    return dim3((unsigned)((K + ACT_THREADS - 1) / ACT_THREADS), (unsigned)(tokens < ACT_MAX_ROWS ? tokens : ACT_MAX_ROWS));
}

}  // namespace

int launch_absmax_f32(const float* X, int tokens, int K, int ldx, float* absmax, hipStream_t st)
{
    begin_launch();
    const bool dense = ldx == K;
    const Rows r = flatten(tokens, K, dense);
    auto blocks = [](long long items) { return dim3((unsigned)(items < (long long)MAX_BLOCKS * MAX_THREADS ? (items + MAX_THREADS - 1) / MAX_THREADS : MAX_BLOCKS)); };
    if ((uintptr_t)X % 16 == 0 && r.K % 4 == 0 && (dense || ldx % 4 == 0)) {
        const long long vecs = r.K / 4, total = vecs * r.tokens;
        if (r.tokens == 1)
            hipLaunchKernelGGL(absmax_vec_kernel<true>, blocks(total), dim3(MAX_THREADS), 0, st, reinterpret_cast<const v4f_t*>(X), total,
                               vecs, 0ll, absmax);
        else
            hipLaunchKernelGGL(absmax_vec_kernel<false>, blocks(total), dim3(MAX_THREADS), 0, st, reinterpret_cast<const v4f_t*>(X), total,
                               vecs, (long long)ldx / 4, absmax);
    } else {
        const long long total = (long long)tokens * K;
        hipLaunchKernelGGL(absmax_any_kernel, blocks(total), dim3(MAX_THREADS), 0, st, X, total, (long long)K, (long long)ldx, absmax);
    }
    return launch_status();
}

int launch_quantize_act(const float* X, int tokens, int K, int ldx, float scale, const float* scale_dev, int8_t* Q, int ldq,
                        hipStream_t st)
{
    begin_launch();
    const bool dense = ldx == K && ldq == K;
    const Rows r = flatten(tokens, K, dense);
    if ((uintptr_t)X % 16 == 0 && (uintptr_t)Q % 4 == 0 && r.K % 4 == 0 && (dense || (ldx % 4 == 0 && ldq % 4 == 0)))
        hipLaunchKernelGGL(quantize_act_vec_kernel, vec_grid(r), dim3(ACT_THREADS), 0, st, reinterpret_cast<const v4f_t*>(X),
                           r.tokens, r.K / 4, (long long)ldx / 4, scale, scale_dev, reinterpret_cast<uint32_t*>(Q),
                           (long long)ldq / 4);
    else
        hipLaunchKernelGGL(quantize_act_any_kernel, any_grid(tokens, K), dim3(ACT_THREADS), 0, st, X, tokens, K, (long long)ldx, scale,
                           scale_dev, Q, (long long)ldq);
    return launch_status();
}

}  // namespace nm
