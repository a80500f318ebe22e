// nm_scale_search: the second scale rule of Sec. 3.3.1 ("ADMM-Dist") on gfx950 - per group of
// output neurons the scale that minimises the squared L2 distance between the kept parameters and
// their quantised values, searched over the candidate grid that the declaration in include/nm.h
// fixes (the paper states the criterion, not an algorithm).
//
// Three launches: the groups' max-rule scales (into the scales array), the error of every
// candidate per row (one wavefront per row, double precision, into the workspace), and per group
// the sum over its rows and the choice.  The per-row partial errors are the only scratch memory:
// [rows][candidates / 2 + 1] doubles.  Sums run in a fixed order (lane-strided partial sums, a fixed
// butterfly over the wavefront, then the rows of a group one after the other), so a call is
// deterministic; it is not the CPU's plain left-to-right order, so candidates whose errors agree
// to about 1e-15 relative can be ranked differently than there.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "nm.h"
#include "nm_internal.h"

// Scratch of the entry point that allocates nothing (nm_scale_search_static): the rows' partial
// errors live in this array instead of a caller's workspace.  Every GPU the library runs on holds
// its own copy, at its own address, until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress - never a device address.
static __device__ __align__(256) unsigned char scratch[NM_SCALE_SEARCH_STATIC_MAX_BYTES];

namespace nm {

namespace {

constexpr int MAX_CAND = 33;                   // candidates / 2 + 1 with candidates <= 64

__device__ __forceinline__ float candidate_scale(float smax, int c, int candidates)
{
    return __fdiv_rn(__fmul_rn(smax, (float)c), (float)candidates);
}

// scales[row] holds the max-rule scale of the row's group.  err[row][k] = sum over the row's kept
// entries of (w - s_k * q_k(w))^2 for candidate k = c - candidates / 2.
template <int M>
__global__ void __launch_bounds__(256)
row_errors_kernel(const float* __restrict__ W, int rows, int cols, int ldw, int N, int bits, int candidates,
                  const float* __restrict__ scales, double* __restrict__ err)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;                   // no barrier below
    const int nc = candidates / 2 + 1;
    const float smax = scales[row];
    const float qmax = (float)((1 << (bits - 1)) - 1);
    double e[MAX_CAND];
#pragma unroll
    for (int k = 0; k < MAX_CAND; ++k) e[k] = 0.0;
    const float* w = W + (size_t)row * ldw;
    for (int g = lane; g < cols / M; g += 64) {
        float v[M], a[M];
#pragma unroll
        for (int c = 0; c < M; ++c) {
            v[c] = w[g * M + c];
            a[c] = fabsf(v[c]);
        }
#pragma unroll
        for (int c = 0; c < M; ++c) {
            // Eq. 3: kept when fewer than N entries outrank it (larger magnitude, or equal and a lower column)
            int outranked = 0;
#pragma unroll
            for (int d = 0; d < M; ++d) {
                if (d == c) continue;
                outranked += (d < c) ? (a[d] >= a[c]) : (a[d] > a[c]);
            }
            if (outranked >= N) continue;
#pragma unroll
            for (int k = 0; k < MAX_CAND; ++k) {
                if (k < nc) {
                    const float s = candidate_scale(smax, candidates / 2 + k, candidates);
                    const float q = fminf(fmaxf(rintf(__fdiv_rn(v[c], s)), -qmax), qmax);      // Eq. 5, offset 0
                    const double d = __dsub_rn((double)v[c], __dmul_rn((double)s, (double)q));
                    e[k] = __dadd_rn(e[k], __dmul_rn(d, d));
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < MAX_CAND; ++k) {
        if (k < nc) {
            double t = e[k];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) t = __dadd_rn(t, __shfl_xor(t, d, 64));
            if (lane == 0) err[(size_t)row * nc + k] = t;
        }
    }
}

// One wavefront per scale group: lane k sums candidate k over the group's rows, then the least
// error wins, the larger scale between equal errors; every row of the group receives the scale.
__global__ void __launch_bounds__(256)
choose_scale_kernel(const double* __restrict__ err, int rows, int rows_per_scale, int candidates, float* __restrict__ scales)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long r0 = ((long long)blockIdx.x * 4 + wave) * rows_per_scale;
    if (r0 >= rows) return;
    const int r1 = (int)((r0 + rows_per_scale < rows) ? r0 + rows_per_scale : rows);
    const int nc = candidates / 2 + 1;
    const float smax = scales[r0];             // read before any row of the group is overwritten (same wavefront)
    double total = 0.0;
    if (lane < nc)
        for (int r = (int)r0; r < r1; ++r) total = __dadd_rn(total, err[(size_t)r * nc + lane]);
    int best = lane < nc ? lane : -1;
    double best_err = total;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const double oe = __shfl_xor(best_err, d, 64);
        const int ob = __shfl_xor(best, d, 64);
        const bool take = ob >= 0 && (best < 0 || oe < best_err || (oe == best_err && ob > best));
        best_err = take ? oe : best_err;
        best = take ? ob : best;
    }
    const float s = candidate_scale(smax, candidates / 2 + best, candidates);
    for (int r = (int)r0 + lane; r < r1; r += 64) scales[r] = s;
}

}  // namespace

int launch_scale_search(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                        int candidates, float* scales, double* row_errors, hipStream_t st)
{
    begin_launch();
    launch_group_scales(W, rows, cols, ldw, rows_per_scale, (float)((1 << (bits - 1)) - 1), scales, st);
    if (M == 4)
        hipLaunchKernelGGL(row_errors_kernel<4>, dim3((rows + 3) / 4), dim3(256), 0, st, W, rows, cols, ldw, N, bits, candidates, scales, row_errors);
    else
        hipLaunchKernelGGL(row_errors_kernel<8>, dim3((rows + 3) / 4), dim3(256), 0, st, W, rows, cols, ldw, N, bits, candidates, scales, row_errors);
    const long long n_groups = ((long long)rows + rows_per_scale - 1) / rows_per_scale;
    hipLaunchKernelGGL(choose_scale_kernel, dim3((unsigned)((n_groups + 3) / 4)), dim3(256), 0, st, row_errors, rows, rows_per_scale, candidates, scales);
    return launch_status();
}

// The device address of `scratch` on the current device, looked up once per device (with that
// device current) and kept.  Returns 0, or NM_ERR_HIP.
static int static_scratch(void** out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex lock;
    static void* address[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        fprintf(stderr, "libnm: nm_scale_search_static: no current device\n");
        return NM_ERR_HIP;
    }
    std::lock_guard<std::mutex> guard(lock);
    if (address[dev] == nullptr) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            fprintf(stderr, "libnm: nm_scale_search_static: hipGetSymbolAddress failed on device %d: %s\n", dev, hipGetErrorString(e));
            return NM_ERR_HIP;
        }
        address[dev] = p;
    }
    *out = address[dev];
    return 0;
}

int launch_scale_search_static(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int rows_per_scale,
                               int candidates, float* scales, hipStream_t st)
{
    void* p = nullptr;
    const int rc = static_scratch(&p);
    if (rc) return rc;
    // Nothing in the array has to start at zero: the second launch writes the partial errors of
    // every row and candidate of this call before the third reads exactly those.
    return launch_scale_search(W, rows, cols, ldw, N, M, bits, rows_per_scale, candidates, scales, static_cast<double*>(p), st);
}

}  // namespace nm
