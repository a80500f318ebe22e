// nm_project: the Z-update of the ADMM decomposition, Z = Pi(W + U) (Sec. 3.1, Eq. 3 applied to
// W + U), with the quantisation constraint solved after the sparsity constraint (Sec. 3.3.1,
// ADMM-Max scale per group of output neurons, Sec. 4) and the dual update U + W - Z, on gfx950.
//
// Purely HBM-bound: 4 (W) + 4 (U) bytes read and 4 (Z) + 4 (U') bytes written per weight, plus
// one more read of W and U for the scales.  Three small kernels, no workspace: the per-row scale
// array the caller passes first receives the rows' largest magnitudes, is then turned in place into
// the scales of the row groups, and is finally read by the projection proper.  Every arithmetic
// step is one fp32 operation, in the order the declaration of nm_project states.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

namespace {

__device__ __forceinline__ float wave_max_f(float m)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    return m;
}

// Largest |W + U| of every row (one wavefront per row, four rows per workgroup).
__global__ void __launch_bounds__(256)
project_amax_kernel(const float* __restrict__ W, const float* __restrict__ U, int rows, int cols, int ldw,
                    float* __restrict__ amax, int vec)         // vec: rows are whole, 16-byte aligned float4s
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;                   // no barrier below
    if (!vec) {                                // any alignment, any width: one float at a time
        float m = 0.0f;
        for (int c = lane; c < cols; c += 64) {
            float v = W[(size_t)row * ldw + c];
            if (U) v = __fadd_rn(v, U[(size_t)row * ldw + c]);
            m = fmaxf(m, fabsf(v));
        }
        m = wave_max_f(m);
        if (lane == 0) amax[row] = m;
        return;
    }
    const float4* __restrict__ w4 = reinterpret_cast<const float4*>(W + (size_t)row * ldw);
    const float4* __restrict__ u4 = U ? reinterpret_cast<const float4*>(U + (size_t)row * ldw) : nullptr;
    float m = 0.0f;
    for (int i = lane; i < cols / 4; i += 64) {
        float4 v = w4[i];
        if (u4) {
            const float4 u = u4[i];
            v.x = __fadd_rn(v.x, u.x); v.y = __fadd_rn(v.y, u.y); v.z = __fadd_rn(v.z, u.z); v.w = __fadd_rn(v.w, u.w);
        }
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    m = wave_max_f(m);
    if (lane == 0) amax[row] = m;
}

// Row maxima -> scales of the row groups, in place: one wavefront per group of rows_per_scale
// rows; s = largest magnitude / largest code (Sec. 3.3.1), 1 for an all-zero group.
__global__ void __launch_bounds__(256)
project_scale_kernel(float* __restrict__ s, int rows, int rows_per_scale, float qmax)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long r0 = ((long long)blockIdx.x * 4 + wave) * rows_per_scale;
    if (r0 >= rows) return;
    const int r1 = (int)((r0 + rows_per_scale < rows) ? r0 + rows_per_scale : rows);
    float m = 0.0f;
    for (int r = (int)r0 + lane; r < r1; r += 64) m = fmaxf(m, s[r]);
    m = wave_max_f(m);
    const float scale = (m == 0.0f) ? 1.0f : __fdiv_rn(m, qmax);
    for (int r = (int)r0 + lane; r < r1; r += 64) s[r] = scale;
}

// Both of the above in one launch for scale groups of moderate size: one workgroup per group of
// rows, its four wavefronts sharing the rows, the largest magnitude combined through LDS.
__global__ void __launch_bounds__(256)
project_group_scale_kernel(const float* __restrict__ W, const float* __restrict__ U, int rows, int cols, int ldw,
                           int rows_per_scale, float qmax, float* __restrict__ s)
{
    __shared__ float part[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long r0 = (long long)blockIdx.x * rows_per_scale;
    const int r1 = (int)((r0 + rows_per_scale < rows) ? r0 + rows_per_scale : rows);
    const int c4 = cols / 4;
    const long long total = (long long)(r1 - (int)r0) * c4;          // 16-byte pieces of the group
    float m = 0.0f;
    for (long long i = threadIdx.x; i < total; i += 256) {
        const int r = (int)r0 + (int)(i / c4), c = (int)(i % c4);
        float4 v = reinterpret_cast<const float4*>(W + (size_t)r * ldw)[c];
        if (U) {
            const float4 u = reinterpret_cast<const float4*>(U + (size_t)r * ldw)[c];
            v.x = __fadd_rn(v.x, u.x); v.y = __fadd_rn(v.y, u.y); v.z = __fadd_rn(v.z, u.z); v.w = __fadd_rn(v.w, u.w);
        }
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    m = wave_max_f(m);
    if (lane == 0) part[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float scale = (m == 0.0f) ? 1.0f : __fdiv_rn(m, qmax);
    for (int r = (int)r0 + threadIdx.x; r < r1; r += 256) s[r] = scale;
}

// One thread per group of M consecutive columns.
template <int M>
__global__ void __launch_bounds__(256)
project_kernel(const float* __restrict__ W, const float* U, int rows, int cols, int ldw,
               int N, int bits, const float* __restrict__ scales,
               float* __restrict__ Z, float* U_out, int ldz)     // U_out may be U (same leading dimension): no restrict on the two
{
    const int groups = cols / M;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)rows * groups) return;
    const int row = (int)(id / groups), g = (int)(id - (long long)row * groups);
    const size_t in_at = (size_t)row * ldw + (size_t)g * M, out_at = (size_t)row * ldz + (size_t)g * M;

    float v[M];
#pragma unroll
    for (int f = 0; f < M / 4; ++f) {
        float4 x = *reinterpret_cast<const float4*>(W + in_at + 4 * f);
        if (U) {
            const float4 u = *reinterpret_cast<const float4*>(U + in_at + 4 * f);
            x.x = __fadd_rn(x.x, u.x); x.y = __fadd_rn(x.y, u.y); x.z = __fadd_rn(x.z, u.z); x.w = __fadd_rn(x.w, u.w);
        }
        v[4 * f + 0] = x.x; v[4 * f + 1] = x.y; v[4 * f + 2] = x.z; v[4 * f + 3] = x.w;
    }
    const float s = bits ? scales[row] : 1.0f;
    const float qmax = (float)((1 << (bits ? bits - 1 : 7)) - 1);
    // Eq. 5 (offset 0), then Eq. 4: the value the integer code stands for (an integer code: its zero has no sign)
    auto requantised = [&](float x) {
        const int q = (int)fminf(fmaxf(rintf(__fdiv_rn(x, s)), -qmax), qmax);
        return __fmul_rn(s, (float)q);
    };
    if constexpr (M == 4) {
        if (N <= 2) {
            // Groups of four with one or two kept: the six pairwise comparisons decide every pair
            // (the lower column outranks on >=, the higher one otherwise), the keep flags follow
            // from them, and only the kept entries (the lowest and the highest kept column) are
            // quantised.
            const float a0 = fabsf(v[0]), a1 = fabsf(v[1]), a2 = fabsf(v[2]), a3 = fabsf(v[3]);
            const bool c01 = a0 >= a1, c02 = a0 >= a2, c03 = a0 >= a3, c12 = a1 >= a2, c13 = a1 >= a3, c23 = a2 >= a3;
            float z0, z1, z2, z3;
            if (N == 2) {
                auto under_two = [](bool p, bool q, bool r) { return !((p && q) || (p && r) || (q && r)); };
                const bool k0 = under_two(!c01, !c02, !c03), k1 = under_two(c01, !c12, !c13);
                const bool k2 = under_two(c02, c12, !c23), k3 = under_two(c03, c13, c23);
                float lo = k0 ? v[0] : (k1 ? v[1] : v[2]);
                float hi = k3 ? v[3] : (k2 ? v[2] : v[1]);
                if (bits) { lo = requantised(lo); hi = requantised(hi); }
                z0 = k0 ? lo : 0.0f;
                z1 = k1 ? (k0 ? hi : lo) : 0.0f;
                z2 = k2 ? (k3 ? lo : hi) : 0.0f;
                z3 = k3 ? hi : 0.0f;
            } else {
                const bool k0 = c01 && c02 && c03, k1 = !c01 && c12 && c13, k2 = !c02 && !c12 && c23;
                const bool k3 = !(k0 || k1 || k2);
                float kept = k0 ? v[0] : (k1 ? v[1] : (k2 ? v[2] : v[3]));
                if (bits) kept = requantised(kept);
                z0 = k0 ? kept : 0.0f; z1 = k1 ? kept : 0.0f; z2 = k2 ? kept : 0.0f; z3 = k3 ? kept : 0.0f;
            }
            *reinterpret_cast<float4*>(Z + out_at) = make_float4(z0, z1, z2, z3);
            if (U_out)
                *reinterpret_cast<float4*>(U_out + out_at) =
                    make_float4(__fsub_rn(v[0], z0), __fsub_rn(v[1], z1), __fsub_rn(v[2], z2), __fsub_rn(v[3], z3));
            return;
        }
    }
    // Eq. 3: an entry is kept when fewer than N entries outrank it; a larger magnitude outranks a
    // smaller one and, between equal magnitudes, the lower column the higher.
    float a[M];
#pragma unroll
    for (int c = 0; c < M; ++c) a[c] = fabsf(v[c]);
    float z[M];
#pragma unroll
    for (int c = 0; c < M; ++c) {
        int outranked = 0;
#pragma unroll
        for (int d = 0; d < M; ++d) {
            if (d == c) continue;
            outranked += (d < c) ? (a[d] >= a[c]) : (a[d] > a[c]);
        }
        float kept_value = v[c];
        if (bits) kept_value = requantised(v[c]);
        z[c] = (outranked < N) ? kept_value : 0.0f;
    }
#pragma unroll
    for (int f = 0; f < M / 4; ++f) {
        *reinterpret_cast<float4*>(Z + out_at + 4 * f) = make_float4(z[4 * f + 0], z[4 * f + 1], z[4 * f + 2], z[4 * f + 3]);
        if (U_out)
            *reinterpret_cast<float4*>(U_out + out_at + 4 * f) =
                make_float4(__fsub_rn(v[4 * f + 0], z[4 * f + 0]), __fsub_rn(v[4 * f + 1], z[4 * f + 1]),
                            __fsub_rn(v[4 * f + 2], z[4 * f + 2]), __fsub_rn(v[4 * f + 3], z[4 * f + 3]));
    }
}

}  // namespace

// scales[row] <- the scale of the row's group: largest |W| over the group's rows / qmax, 1 for an
// all-zero group.  Two launches, no workspace (scales[] first holds the rows' maxima).
void launch_group_scales(const float* W, int rows, int cols, int ldw, int rows_per_scale, float qmax, float* scales,
                         hipStream_t st)
{
    const int vec = ((uintptr_t)W % 16 == 0 && ldw % 4 == 0 && cols % 4 == 0) ? 1 : 0;
    hipLaunchKernelGGL(project_amax_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, W, (const float*)nullptr, rows, cols, ldw, scales, vec);
    const long long n_groups = ((long long)rows + rows_per_scale - 1) / rows_per_scale;
    hipLaunchKernelGGL(project_scale_kernel, dim3((unsigned)((n_groups + 3) / 4)), dim3(256), 0, st, scales, rows, rows_per_scale, qmax);
}

int launch_project(const float* W, const float* U, int rows, int cols, int ldw, int N, int M, int bits,
                   int rows_per_scale, float* Z, float* U_out, int ldz, float* scales, hipStream_t st)
{
    begin_launch();
    if (bits) {
        const float qmax = (float)((1 << (bits - 1)) - 1);
        const long long n_groups = ((long long)rows + rows_per_scale - 1) / rows_per_scale;
        // A workgroup per scale group reads the group alone: fine while a group is a row or a few
        // (3072 x 768, one row per scale: 10.4 against 11.7 us); for 32 rows per scale the 96
        // workgroups that remain are too few to pull the matrix in (20.6 against 14.0 us), so then
        // row maxima first, all rows at once, and the groups in a second small launch.
        if (n_groups >= 512 && (long long)rows_per_scale * cols <= 4096) {
            hipLaunchKernelGGL(project_group_scale_kernel, dim3((unsigned)n_groups), dim3(256), 0, st,
                               W, U, rows, cols, ldw, rows_per_scale, qmax, scales);
        } else {
            hipLaunchKernelGGL(project_amax_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, W, U, rows, cols, ldw, scales, 1);
            hipLaunchKernelGGL(project_scale_kernel, dim3((unsigned)((n_groups + 3) / 4)), dim3(256), 0, st,
                               scales, rows, rows_per_scale, qmax);
        }
    }
    const long long total = (long long)rows * (cols / M);
    const dim3 grid((unsigned)((total + 255) / 256));
    if (M == 4)
        hipLaunchKernelGGL(project_kernel<4>, grid, dim3(256), 0, st, W, U, rows, cols, ldw, N, bits, scales, Z, U_out, ldz);
    else
        hipLaunchKernelGGL(project_kernel<8>, grid, dim3(256), 0, st, W, U, rows, cols, ldw, N, bits, scales, Z, U_out, ldz);
    return launch_status();
}

}  // namespace nm
