// nm_compress / nm_decompress_i8 kernels for gfx950.
//
// nm_compress applies, per output row, the N:M projection of Sec. 3.2 (Eq. 3), the
// max-rule scale of Sec. 3.3.1 and the symmetric quantiser of Sec. 3.3 (Eq. 5, offset 0),
// in that order (Sec. 3.3.1, last paragraph), and writes the packed format described in
// include/nm.h.  The work is bound by reading the fp32 matrix once from HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "nm_quantize.h"

namespace nm {

namespace {

// Lane-crossing moves inside a row of 16 lanes through the DPP path of the vector ALU (no LDS
// round trip): controls 0xB1 / 0x4E swap neighbours at distance 1 / 2 inside each quad, 0x141
// mirrors each half-row of 8, 0x140 mirrors the row of 16.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

// max over the 64 lanes, result in every lane
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, __uint_as_float(dpp_u32<0xB1>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_u32<0x4E>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_u32<0x141>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_u32<0x140>(__float_as_uint(v))));
    const int b = (int)__float_as_uint(v);               // every lane now holds its row's maximum
    const float r0 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(b, 0));
    const float r1 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(b, 16));
    const float r2 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(b, 32));
    const float r3 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// OR together the LANES consecutive lanes of each aligned lane group (LANES = 1, 2, 4, 8 or 16).
template <int LANES>
__device__ __forceinline__ uint32_t group_or(uint32_t v)
{
    static_assert(LANES == 1 || LANES == 2 || LANES == 4 || LANES == 8 || LANES == 16, "group within a row of 16");
    if constexpr (LANES >= 2) v |= dpp_u32<0xB1>(v);
    if constexpr (LANES >= 4) v |= dpp_u32<0x4E>(v);
    if constexpr (LANES >= 8) v |= dpp_u32<0x141>(v);
    if constexpr (LANES >= 16) v |= dpp_u32<0x140>(v);
    return v;
}

// Eq. 3 on one group held in registers.  Returns a bit mask of the kept columns: an entry is
// kept when fewer than N entries outrank it, where a larger magnitude outranks a smaller one
// and, between equal magnitudes, the lower column outranks the higher.
template <int N, int M>
__device__ __forceinline__ uint32_t keep_mask(const float (&x)[M])
{
    float a[M];
#pragma unroll
    for (int c = 0; c < M; ++c) a[c] = fabsf(x[c]);
    uint32_t mask = 0;
#pragma unroll
    for (int c = 0; c < M; ++c) {
        int outranked = 0;
#pragma unroll
        for (int d = 0; d < M; ++d) {
            if (d == c) continue;
            outranked += (d < c) ? (a[d] >= a[c]) : (a[d] > a[c]);
        }
        mask |= (outranked < N ? 1u : 0u) << c;
    }
    return mask;
}

// One group -> its value bits (N codes of BITS bits, ascending columns) and index bits.  Kept
// column c goes to slot (number of kept columns below c); every register is addressed with a
// compile-time index so the group never leaves the register file.
template <int N, int M, int BITS, bool RECIP>
__device__ __forceinline__ void encode_group(const float (&x)[M], const Divisor<RECIP>& s, uint32_t& vbits, uint32_t& mbits)
{
    constexpr int IB = (M == 4) ? 2 : 4;
    if constexpr (N == M) {
        // dense matrix: every entry is kept, in column order; there are no index bits
        vbits = 0;
        mbits = 0;
#pragma unroll
        for (int j = 0; j < N; ++j) vbits |= ((uint32_t)quantize<BITS>(x[j], s) & ((1u << BITS) - 1u)) << (j * BITS);
        return;
    }
    if constexpr (M == 4 && (N == 1 || N == 2)) {
        // Groups of four, the same rule spelled out: the six comparisons "the lower column is at
        // least as large" decide every pair (the lower column outranks on >=, the higher one
        // otherwise), and with exactly N columns kept the slots follow from the keep flags alone.
        // The flags are wavefront masks combined on the scalar unit; the vector ALU only compares
        // and selects.
        const float a0 = fabsf(x[0]), a1 = fabsf(x[1]), a2 = fabsf(x[2]), a3 = fabsf(x[3]);
        const bool c01 = a0 >= a1, c02 = a0 >= a2, c03 = a0 >= a3, c12 = a1 >= a2, c13 = a1 >= a3, c23 = a2 >= a3;
        if constexpr (N == 2) {
            auto under_two = [](bool p, bool q, bool r) { return !((p && q) || (p && r) || (q && r)); };
            const bool k0 = under_two(!c01, !c02, !c03);       // outranked by fewer than two
            const bool k1 = under_two(c01, !c12, !c13);
            const bool k2 = under_two(c02, c12, !c23);
            const bool k3 = under_two(c03, c13, c23);
            const float lo = k0 ? x[0] : (k1 ? x[1] : x[2]);   // lowest kept column: 0, else 1, else 2
            const uint32_t clo = k0 ? 0u : (k1 ? 1u : 2u);
            const float hi = k3 ? x[3] : (k2 ? x[2] : x[1]);   // highest kept column: 3, else 2, else 1
            const uint32_t chi = k3 ? 3u : (k2 ? 2u : 1u);
            const int q0 = quantize<BITS>(lo, s), q1 = quantize<BITS>(hi, s);
            vbits = ((uint32_t)q0 & ((1u << BITS) - 1u)) | (((uint32_t)q1 & ((1u << BITS) - 1u)) << BITS);
            mbits = clo | (chi << IB);
        } else {
            const bool k0 = c01 && c02 && c03, k1 = !c01 && c12 && c13, k2 = !c02 && !c12 && c23;   // outranked by none
            const float v = k0 ? x[0] : (k1 ? x[1] : (k2 ? x[2] : x[3]));
            mbits = k0 ? 0u : (k1 ? 1u : (k2 ? 2u : 3u));
            vbits = (uint32_t)quantize<BITS>(v, s) & ((1u << BITS) - 1u);
        }
        return;
    }
    if constexpr (M == 8 && (N == 1 || N == 2)) {
        // Groups of eight, one or two kept: each of the 28 pairs is compared once (ge[d][c], d < c:
        // the lower column is at least as large, so it outranks the higher one; otherwise the
        // higher one outranks it), a column's count of outranking entries is the number of
        // columns above it, plus the pairs it loses to lower columns, minus the pairs it wins
        // against higher ones; the slots are the first and the last kept column.
        float a[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) a[c] = fabsf(x[c]);
        bool keep[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            int outranked = 7 - c;
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                if (d < c) outranked += (a[d] >= a[c]) ? 1 : 0;
                if (d > c) outranked -= (a[c] >= a[d]) ? 1 : 0;
            }
            keep[c] = outranked < N;
        }
        float lo = x[7];
        uint32_t clo = 7u;
#pragma unroll
        for (int c = 6; c >= 0; --c) {                  // first kept column
            lo = keep[c] ? x[c] : lo;
            clo = keep[c] ? (uint32_t)c : clo;
        }
        vbits = (uint32_t)quantize<BITS>(lo, s) & ((1u << BITS) - 1u);
        mbits = clo;
        if constexpr (N == 2) {
            float hi = x[0];
            uint32_t chi = 0u;
#pragma unroll
            for (int c = 1; c < 8; ++c) {               // last kept column
                hi = keep[c] ? x[c] : hi;
                chi = keep[c] ? (uint32_t)c : chi;
            }
            vbits |= ((uint32_t)quantize<BITS>(hi, s) & ((1u << BITS) - 1u)) << BITS;
            mbits |= chi << IB;
        }
        return;
    }
    const uint32_t mask = keep_mask<N, M>(x);
    vbits = 0;
    mbits = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        float v = 0.0f;
        uint32_t col = 0;
#pragma unroll
        for (int c = j; c <= M - N + j; ++c) {          // slot j can only hold columns j .. M-N+j
            const bool here = ((mask >> c) & 1u) && (__builtin_popcount(mask & ((1u << c) - 1u)) == j);
            v = here ? x[c] : v;
            col = here ? (uint32_t)c : col;
        }
        const int q = quantize<BITS>(v, s);
        vbits |= ((uint32_t)q & ((1u << BITS) - 1u)) << (j * BITS);
        mbits |= col << (j * IB);
    }
}

// ---------------------------------------------------------------------------------------------
// WPR wavefronts per row (1, 2 or 4; four wavefronts per workgroup).  Pass p of a row covers
// groups 64p .. 64p+63, lane l owning group 64p + l, so the fp32 row is read with lane-contiguous
// 16-byte loads; wavefront w of the row takes passes w, w+WPR, ...  The per-group value / index
// bits of neighbouring lanes are OR-combined into whole dwords before they are stored.  A
// wavefront keeps up to 64 floats per lane in registers between the amax pass and the encode
// pass (rows up to 4096*WPR columns); longer rows are read a second time.  Long rows are split
// over several wavefronts because one wavefront walking a 3072-wide row alone is bound by its own
// serial arithmetic, not by memory.
// Requires: N*BITS and N*IB in {2,4,8,16,32}, packed row strides that are multiples of 4 bytes,
// ldw % 4 == 0 and a 16-byte aligned W.
// ---------------------------------------------------------------------------------------------
// The fp32 weights are read once and never again.  A batched call whose matrices exceed what the L2s
// hold together (32 MB) loads them with the streaming hint, so that they do not push the operands of the
// GEMMs that follow out of the caches (the 48 matrices of a 12-layer encoder, 340 MB: the GEMMs after
// them 5 % faster; BERT-large's layer set, 50 MB: 2 %); smaller calls use plain loads (a caller that
// compresses the same 28 MB again and again finds them in the Infinity Cache).
constexpr long long STREAM_ABOVE_BYTES = 32ll << 20;
constexpr int GIVEN_SCALES = 1;                        // bits of the kernels' `flags` argument
constexpr int TILED_LAYOUT = 2;
typedef float v4f_t __attribute__((ext_vector_type(4)));
template <bool ONCE>
__device__ __forceinline__ float4 load_w(const float4* p)
{
    if constexpr (!ONCE) return *p;
    const v4f_t v = __builtin_nontemporal_load(reinterpret_cast<const v4f_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// Byte offset, in the tiled layout, of byte b of a packed row (UB = bytes per unit, a compile-time
// constant here so that the divisions are shifts and multiplications).
template <int UB>
__device__ __forceinline__ uint32_t tiled_at(uint32_t row, uint32_t b, uint32_t slices)
{
    constexpr uint32_t PB = (uint32_t)piece_bytes(UB);
    const uint32_t u = b / UB, i = b % UB;
    return ((row >> 4) * slices + (u >> 2)) * (64u * UB) + ((i / PB) * 64u + (u & 3u) * 16u + (row & 15u)) * PB + i % PB;
}

// One dword of a packed row (dword index `d` of the row layout) to either layout.  In the tiled
// layout a dword lies inside one piece of a unit when pieces are 4 bytes or more; 2-byte pieces
// (units of 2 bytes: a dword spans two units, 16 rows apart) are stored as two halves.
template <int UB>
__device__ __forceinline__ void store_packed(uint8_t* __restrict__ base, int tiled, uint32_t row, uint32_t d,
                                             uint32_t stride_dw, uint32_t slices, uint32_t v)
{
    if (!tiled) {
        reinterpret_cast<uint32_t*>(base)[(size_t)row * stride_dw + d] = v;
        return;
    }
    if constexpr (piece_bytes(UB) >= 4) {
        *reinterpret_cast<uint32_t*>(base + tiled_at<UB>(row, 4u * d, slices)) = v;
    } else {
        *reinterpret_cast<uint16_t*>(base + tiled_at<UB>(row, 4u * d, slices)) = (uint16_t)v;
        *reinterpret_cast<uint16_t*>(base + tiled_at<UB>(row, 4u * d + 2u, slices)) = (uint16_t)(v >> 16);
    }
}

// The rows of one workgroup: `block` is the workgroup's index among those of this matrix, WPR
// (1, 2 or 4) a compile-time constant in the single-matrix kernel and a per-matrix value in the
// batched one (uniform over the workgroup, so the barrier below is too).
template <int N, int M, int BITS, int RES, bool ONCE>
__device__ __forceinline__ void
compress_rows(const float* __restrict__ W, int rows, int cols, int ldw,
              uint32_t* __restrict__ vals, uint32_t* __restrict__ meta, float* __restrict__ scales,
              int vstride_dw, int mstride_dw, int flags, const int WPR, const int block, float* part)
{
    const bool given = (flags & GIVEN_SCALES) != 0;
    const int tiled = (flags & TILED_LAYOUT) ? 1 : 0;
    constexpr bool HAS_META = N < M;       // a dense matrix stores no index bits
    constexpr int IB = (M == 4) ? 2 : 4;
    constexpr int VB = N * BITS;           // value bits per group
    constexpr int MB = HAS_META ? N * IB : 32;   // index bits per group
    constexpr int VL = 32 / VB;            // lanes per value dword
    constexpr int ML = 32 / MB;            // lanes per index dword
    constexpr int UV = 32 / M * N * BITS / 8;    // packed value / index bytes per 32 input columns
    constexpr int UM = HAS_META ? 32 / M * N * IB / 8 : 4;
    constexpr int F4 = M / 4;              // 16-byte loads per group
    static_assert(RES * F4 <= 16, "at most 64 floats per lane stay in registers");
    const int RPB = 4 / WPR;               // rows per workgroup
    constexpr float QMAX = (float)((1 << (BITS - 1)) - 1);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // the row and the wavefront's place in it are the same in all lanes: said so explicitly, the row's
    // base addresses stay in scalar registers and every access is base + 32-bit lane offset
    const int row_raw = __builtin_amdgcn_readfirstlane(block * RPB + wave / WPR);
    const bool live = row_raw < rows;      // rows past the end are computed on the last row and not stored ...
    const int row = live ? row_raw : rows - 1;
    // ... except that the tiled layout pads the rows to a multiple of 16 with zero bytes
    const bool store = live || (tiled && row_raw < ((rows + 15) & ~15));
    const uint32_t slices = (uint32_t)cols >> 7;
    const int w = __builtin_amdgcn_readfirstlane(wave % WPR);

    const float4* __restrict__ w4 = reinterpret_cast<const float4*>(W + (size_t)row * ldw);
    const int groups = cols / M;
    const int passes = (groups + 63) >> 6;                 // of the whole row
    const int mine = (passes - w + WPR - 1) / WPR;          // passes of this wavefront: w, w+WPR, ...
    const bool resident = mine <= RES;

    float4 x[RES * F4];                     // only ever indexed with compile-time constants: stays in registers
#pragma unroll
    for (int i = 0; i < RES * F4; ++i) x[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float amax = 0.0f;
    if (resident) {
#pragma unroll
        for (int i = 0; i < RES; ++i) {
            const int g = (w + i * WPR) * 64 + lane;
            if (i < mine && g < groups) {
#pragma unroll
                for (int f = 0; f < F4; ++f) x[i * F4 + f] = load_w<ONCE>(w4 + (unsigned)(g * F4 + f));
            }
        }
#pragma unroll
        for (int i = 0; i < RES * F4; ++i) {
            const float4 v = x[i];
            amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
    } else {
        for (int i = 0; i < mine; ++i) {
            const int g = (w + i * WPR) * 64 + lane;
            if (g < groups)
#pragma unroll
                for (int f = 0; f < F4; ++f) {
                    float4 v = load_w<ONCE>(w4 + (unsigned)(g * F4 + f));
                    amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
                }
        }
    }
    amax = wave_max(amax);
    if (WPR > 1) {
        if (lane == 0) part[wave] = amax;
        __syncthreads();
        const int first = (wave / WPR) * WPR;
        amax = part[first];
        for (int k = 1; k < WPR; ++k) amax = fmaxf(amax, part[first + k]);
    }
    // Sec. 3.3.1: largest magnitude over the largest code; an all-zero row keeps scale 1
    // (the same value in every lane of the row's wavefronts: kept in a scalar register)
    const float s = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane(
        (int)__float_as_uint(given ? scales[row] : ((amax == 0.0f) ? 1.0f : amax / QMAX))));
    if (!given && live && w == 0 && lane == 0) scales[row] = s;

    uint8_t* __restrict__ vbase = reinterpret_cast<uint8_t*>(vals);
    uint8_t* __restrict__ mbase = reinterpret_cast<uint8_t*>(meta);

    auto encode_row = [&](auto divisor) __attribute__((always_inline)) {
        auto emit = [&](const float (&grp)[M], int g) __attribute__((always_inline)) {
            uint32_t vb = 0, mb = 0;
            if (g < groups) encode_group<N, M, BITS>(grp, divisor, vb, mb);
            vb = group_or<VL>(vb << ((lane % VL) * VB));
            if (store && g < groups && lane % VL == 0)
                store_packed<UV>(vbase, tiled, (uint32_t)row_raw, (uint32_t)g / VL, (uint32_t)vstride_dw, slices, live ? vb : 0u);
            if constexpr (HAS_META) {
                mb = group_or<ML>(mb << ((lane % ML) * MB));
                if (store && g < groups && lane % ML == 0)
                    store_packed<UM>(mbase, tiled, (uint32_t)row_raw, (uint32_t)g / ML, (uint32_t)mstride_dw, slices, live ? mb : 0u);
            }
        };
        if (resident) {
#pragma unroll
            for (int i = 0; i < RES; ++i) {
                if (i < mine) {
                    float grp[M];
#pragma unroll
                    for (int f = 0; f < F4; ++f) {
                        const float4 v = x[i * F4 + f];
                        grp[4 * f + 0] = v.x; grp[4 * f + 1] = v.y; grp[4 * f + 2] = v.z; grp[4 * f + 3] = v.w;
                    }
                    emit(grp, (w + i * WPR) * 64 + lane);
                }
            }
        } else {
            for (int i = 0; i < mine; ++i) {
                const int g = (w + i * WPR) * 64 + lane;
                float grp[M];
#pragma unroll
                for (int f = 0; f < F4; ++f) {
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (g < groups) v = load_w<ONCE>(w4 + (unsigned)(g * F4 + f));
                    grp[4 * f + 0] = v.x; grp[4 * f + 1] = v.y; grp[4 * f + 2] = v.z; grp[4 * f + 3] = v.w;
                }
                emit(grp, g);
            }
        }
    };
    // One division per row (the reciprocal) instead of one per kept weight wherever the scale is
    // in the range for which that route is exact; any other scale takes the division operator.
    if (s >= 0x1p-60f && s <= 0x1p60f) encode_row(Divisor<true>{s, __fdiv_rn(1.0f, s)});
    else encode_row(Divisor<false>{s, 0.0f});
}

// Workgroup -> its share of the rows.  Consecutive workgroups of a launch go to different XCDs
// (eight, each with an L2 of its own).  In the tiled layout the 16 rows of a block share every
// 128-byte line of the output, so the workgroups that write one block must sit on one XCD for the
// line to leave its L2 whole instead of in eight masked pieces: workgroup i of n (n a multiple of
// 8) takes share (i % 8) * (n / 8) + i / 8, which gives every XCD one contiguous range of rows.
__device__ __forceinline__ int xcd_block(int i, int n, int flags)
{
    return (flags & TILED_LAYOUT) ? (i & 7) * (n >> 3) + (i >> 3) : i;
}

template <int N, int M, int BITS, int WPR, int RES>
__global__ void __launch_bounds__(256)
compress_wave_kernel(const float* __restrict__ W, int rows, int cols, int ldw,
                     uint32_t* __restrict__ vals, uint32_t* __restrict__ meta, float* __restrict__ scales,
                     int vstride_dw, int mstride_dw, int flags)      // GIVEN_SCALES: scales[] holds the rows' scales already
{
    __shared__ float part[4];
    compress_rows<N, M, BITS, RES, false>(W, rows, cols, ldw, vals, meta, scales, vstride_dw, mstride_dw, flags, WPR,
                                          xcd_block((int)blockIdx.x, (int)gridDim.x, flags), part);
}

// Several matrices of one pattern in one launch: the descriptors travel by value in the kernel
// arguments (no device table to allocate or copy), each matrix owns a contiguous range of
// workgroups.  What a launch costs beside its bytes (a few microseconds: start-up, the latency of
// the first loads, the drain) is then paid once for a layer's weight matrices, not once per matrix.
constexpr int BATCH_MAX = 16;
struct BatchItem {
    const float* W;
    uint32_t* vals;
    uint32_t* meta;
    float* scales;
    int rows, cols, ldw, vstride_dw, mstride_dw, wpr, first_block, blocks;
};
struct BatchArgs {
    // the table a workgroup searches for its item, one aligned 64-byte run at the front of the
    // argument block so that it arrives in one scalar load; unused entries hold INT_MAX
    int first_block[BATCH_MAX];
    int count;
    int flags;             // of compress_rows
    int stream_loads;      // the weights are loaded with the streaming hint
    BatchItem it[BATCH_MAX];
};

template <int N, int M, int BITS, int RES, bool ONCE>
__global__ void __launch_bounds__(256)
compress_batch_kernel(const BatchArgs b)
{
    __shared__ float part[4];
    // Two round trips to the argument memory before the first weights are asked for: the table,
    // then every field of the item at once (fetched where first used they were four to seven).
    int i = 0;
#pragma unroll
    for (int k = 1; k < BATCH_MAX; ++k)
        if ((int)blockIdx.x >= b.first_block[k]) i = k;        // uniform
    BatchItem t = b.it[i];
    asm volatile("" : "+s"(t.W), "+s"(t.vals), "+s"(t.meta), "+s"(t.scales), "+s"(t.rows), "+s"(t.cols), "+s"(t.ldw),
                      "+s"(t.vstride_dw), "+s"(t.mstride_dw), "+s"(t.wpr), "+s"(t.first_block), "+s"(t.blocks));
    compress_rows<N, M, BITS, RES, ONCE>(t.W, t.rows, t.cols, t.ldw, t.vals, t.meta, t.scales, t.vstride_dw, t.mstride_dw, b.flags,
                                   t.wpr, xcd_block((int)blockIdx.x - t.first_block, t.blocks, b.flags), part);
}

// ---------------------------------------------------------------------------------------------
// The patterns whose groups do not pack into whole fractions of a dword (3:4, 3:8, 5:8, 6:8, 7:8:
// 6 to 56 value bits and 6 to 28 index bits per group): a wavefront per row, four rows per
// workgroup.  Lane l encodes groups l, l + 64, ... as the kernels above do (same ranking, same
// quantiser) and ORs each group's bits into the row's image in LDS at their bit offset, wherever
// that falls in a dword; the image then goes out in dwords, to either layout.  Needs a 16-byte
// aligned W, ldw % 4 == 0 and packed rows of whole dwords.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void or_bits(uint32_t* image, uint32_t bit, uint64_t v)     // v < 2^56
{
    const uint32_t d = bit >> 5, sh = bit & 31u;
    const uint64_t lo = v << sh;
    const uint32_t hi = sh ? (uint32_t)(v >> (64u - sh)) : 0u;      // what the shift pushed past 64 bits
    if ((uint32_t)lo) atomicOr(&image[d], (uint32_t)lo);            // (a zero part may lie past the row's end)
    if ((uint32_t)(lo >> 32)) atomicOr(&image[d + 1], (uint32_t)(lo >> 32));
    if (hi) atomicOr(&image[d + 2], hi);
}

template <int N, int M, int BITS>
__global__ void __launch_bounds__(256)
compress_rowimage_kernel(const float* __restrict__ W, int rows, int cols, int ldw,
                         uint8_t* __restrict__ vals, uint8_t* __restrict__ meta, float* __restrict__ scales,
                         PackedArray pv, PackedArray pm, int given)
{
    constexpr int IB = (M == 4) ? 2 : 4;
    constexpr int VB = N * BITS, MB = N * IB;          // value / index bits per group
    constexpr int F4 = M / 4;
    constexpr float QMAX = (float)((1 << (BITS - 1)) - 1);
    extern __shared__ uint32_t images[];               // per wavefront: value dwords, then index dwords, of one row

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    const int rows_out = pv.tiled ? ((rows + 15) & ~15) : rows;     // the tiled layout pads the rows with zero bytes
    if (row >= rows_out) return;                       // (no workgroup-wide barrier below)
    const int vdw = (int)pv.stride / 4, mdw = (int)pm.stride / 4;
    uint32_t* vimg = images + wave * (vdw + mdw);
    uint32_t* mimg = vimg + vdw;
    for (int d = lane; d < vdw + mdw; d += 64) vimg[d] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    if (row < rows) {
        const float4* __restrict__ w4 = reinterpret_cast<const float4*>(W + (size_t)row * ldw);
        const int groups = cols / M;
        float s;
        if (given) {
            s = scales[row];
        } else {
            float amax = 0.0f;
            for (int i = lane; i < groups * F4; i += 64) {
                const float4 v = w4[i];
                amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            }
            amax = wave_max(amax);
            s = (amax == 0.0f) ? 1.0f : amax / QMAX;   // Sec. 3.3.1; an all-zero row keeps scale 1
            if (lane == 0) scales[row] = s;
        }
        auto encode_row = [&](auto divisor) __attribute__((always_inline)) {
            for (int g = lane; g < groups; g += 64) {
                float x[M];
#pragma unroll
                for (int f = 0; f < F4; ++f) {
                    const float4 v = w4[g * F4 + f];
                    x[4 * f + 0] = v.x; x[4 * f + 1] = v.y; x[4 * f + 2] = v.z; x[4 * f + 3] = v.w;
                }
                const uint32_t mask = keep_mask<N, M>(x);
                uint64_t vbits = 0;
                uint32_t mbits = 0;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    float v = 0.0f;
                    uint32_t col = 0;
#pragma unroll
                    for (int c = j; c <= M - N + j; ++c) {          // slot j can only hold columns j .. M-N+j
                        const bool here = ((mask >> c) & 1u) && (__builtin_popcount(mask & ((1u << c) - 1u)) == j);
                        v = here ? x[c] : v;
                        col = here ? (uint32_t)c : col;
                    }
                    const int q = quantize<BITS>(v, divisor);
                    vbits |= (uint64_t)((uint32_t)q & ((1u << BITS) - 1u)) << (j * BITS);
                    mbits |= col << (j * IB);
                }
                or_bits(vimg, (uint32_t)g * VB, vbits);
                or_bits(mimg, (uint32_t)g * MB, (uint64_t)mbits);
            }
        };
        if (s >= 0x1p-60f && s <= 0x1p60f) encode_row(Divisor<true>{s, __fdiv_rn(1.0f, s)});
        else encode_row(Divisor<false>{s, 0.0f});
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // the image, a dword at a time; in the tiled layout a dword lies inside one piece of a unit when
    // the pieces are 4 bytes or more, and is two pieces (of two different units or halves) otherwise
    auto copy_out = [&](const uint32_t* img, int ndw, uint8_t* base, const PackedArray& pa) __attribute__((always_inline)) {
        const bool halves = pa.tiled && piece_bytes((int)pa.ub) < 4;
        for (int d = lane; d < ndw; d += 64) {
            const uint32_t v = *reinterpret_cast<const volatile uint32_t*>(img + d);
            if (!halves) {
                *reinterpret_cast<uint32_t*>(base + pa.at((uint32_t)row, 4u * d)) = v;
            } else {
                *reinterpret_cast<uint16_t*>(base + pa.at((uint32_t)row, 4u * d)) = (uint16_t)v;
                *reinterpret_cast<uint16_t*>(base + pa.at((uint32_t)row, 4u * d + 2u)) = (uint16_t)(v >> 16);
            }
        }
    };
    copy_out(vimg, vdw, vals, pv);
    copy_out(mimg, mdw, meta, pm);
}

// ---------------------------------------------------------------------------------------------
// Any pattern, any width, any alignment, either layout: one thread per row, bytes written one at
// a time.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64)
compress_generic_kernel(const float* __restrict__ W, int rows, int cols, int ldw, int N, int M, int bits,
                        uint8_t* __restrict__ vals, uint8_t* __restrict__ meta, float* __restrict__ scales,
                        PackedArray pv, PackedArray pm, int given)
{
    const int row = blockIdx.x * 64 + threadIdx.x;
    if (row >= rows) {
        // rows that only pad the tiled layout to a multiple of 16: zero bytes
        if (pv.tiled && row < ((rows + 15) & ~15)) {
            for (uint32_t b = 0; b < pv.stride; ++b) vals[pv.at((uint32_t)row, b)] = 0;
            if (pm.ub)
                for (uint32_t b = 0; b < pm.stride; ++b) meta[pm.at((uint32_t)row, b)] = 0;
        }
        return;
    }
    const float* w = W + (size_t)row * ldw;
    const int ib = (N >= M) ? 0 : (M == 4) ? 2 : 4;
    const int qmaxi = (1 << (bits - 1)) - 1;
    float amax = 0.0f;
    for (int c = 0; c < cols; ++c) amax = fmaxf(amax, fabsf(w[c]));
    const float s = given ? scales[row] : ((amax == 0.0f) ? 1.0f : amax / (float)qmaxi);
    if (!given) scales[row] = s;
    uint32_t vacc = 0, macc = 0;
    int vfill = 0, mfill = 0;
    uint32_t vpos = 0, mpos = 0;
    for (int g = 0; g < cols / M; ++g) {
        float x[8];
        for (int c = 0; c < 8; ++c) x[c] = (c < M) ? w[g * M + c] : 0.0f;
        for (int c = 0; c < M; ++c) {
            int outranked = 0;
            for (int d = 0; d < M; ++d) {
                if (d == c) continue;
                float ad = fabsf(x[d]), ac = fabsf(x[c]);
                outranked += (d < c) ? (ad >= ac) : (ad > ac);
            }
            if (outranked >= N) continue;
            float r = rintf(x[c] / s);
            r = fminf(fmaxf(r, (float)-qmaxi), (float)qmaxi);
            vacc |= ((uint32_t)(int)r & ((1u << bits) - 1u)) << vfill;
            vfill += bits;
            macc |= (uint32_t)c << mfill;
            mfill += ib;
            while (vfill >= 8) { vals[pv.at((uint32_t)row, vpos++)] = (uint8_t)vacc; vacc >>= 8; vfill -= 8; }
            while (mfill >= 8) { meta[pm.at((uint32_t)row, mpos++)] = (uint8_t)macc; macc >>= 8; mfill -= 8; }
        }
    }
    if (vfill > 0) vals[pv.at((uint32_t)row, vpos)] = (uint8_t)vacc;
    if (mfill > 0) meta[pm.at((uint32_t)row, mpos)] = (uint8_t)macc;
}

// Packed -> dense int8, one thread per (row, group).
__global__ void __launch_bounds__(256)
decompress_kernel(const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int rows, int cols,
                  int N, int M, int bits, PackedArray pv, PackedArray pm, int8_t* __restrict__ Wq)
{
    const int groups = cols / M;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)rows * groups) return;
    const int row = (int)(id / groups), g = (int)(id % groups);
    const int ib = (N >= M) ? 0 : (M == 4) ? 2 : 4;
    int8_t out[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = 0; j < N; ++j) {
        const uint32_t e = (uint32_t)(g * N + j);
        int q, off;
        if (bits == 8) q = (int8_t)vals[pv.at((uint32_t)row, e)];
        else { int nib = (vals[pv.at((uint32_t)row, e >> 1)] >> ((e & 1) * 4)) & 15; q = (nib ^ 8) - 8; }
        if (ib == 0) off = j;
        else if (ib == 2) off = (meta[pm.at((uint32_t)row, e >> 2)] >> ((e & 3) * 2)) & 3;
        else off = (meta[pm.at((uint32_t)row, e >> 1)] >> ((e & 1) * 4)) & 15;
        out[off & 7] = (int8_t)q;
    }
    int8_t* dst = Wq + (size_t)row * cols + (size_t)g * M;
    for (int c = 0; c < M; ++c) dst[c] = out[c];
}

// One packed array from one layout to the other, a byte per thread; rows that only pad the tiled
// layout to a multiple of 16 are written as zeros.
__global__ void __launch_bounds__(256)
repack_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int rows, int rows_out, PackedArray ps, PackedArray pd)
{
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)rows_out * ps.stride) return;
    const uint32_t row = (uint32_t)(id / ps.stride), b = (uint32_t)(id % ps.stride);
    dst[pd.at(row, b)] = (row < (uint32_t)rows) ? src[ps.at(row, b)] : (uint8_t)0;
}

template <int N, int M, int BITS, int WPR, int RES>
void launch_wave_res(const float* W, int rows, int cols, int ldw, uint32_t* v, uint32_t* m, float* scales,
                     int vstride, int mstride, int flags, hipStream_t st)
{
    constexpr int RPB = 4 / WPR;
    const int rows_out = (flags & TILED_LAYOUT) ? ((rows + 15) & ~15) : rows;      // the tiled layout pads the rows
    int blocks = (rows_out + RPB - 1) / RPB;
    if (flags & TILED_LAYOUT) blocks = (blocks + 7) & ~7;      // whole rounds over the XCDs, see xcd_block
    hipLaunchKernelGGL((compress_wave_kernel<N, M, BITS, WPR, RES>), dim3(blocks), dim3(256), 0, st,
                       W, rows, cols, ldw, v, m, scales, vstride / 4, mstride / 4, flags);
}

// WPR = wavefronts per row: enough that a wavefront walks at most ~4 passes of 64 groups.  RES =
// passes a wavefront keeps in registers: the smallest compiled size that holds its share of the
// row (the loops over passes unroll completely, so an oversized RES costs instructions for
// nothing); rows too long for the largest size are read twice.
template <int N, int M, int BITS, int WPR>
void launch_wave_wpr(const float* W, int rows, int cols, int ldw, uint32_t* v, uint32_t* m, float* scales,
                     int vstride, int mstride, int flags, hipStream_t st)
{
    constexpr int MAXRES = 16 / (M / 4);
    const int passes = (cols / M + 63) / 64;
    const int mine = (passes + WPR - 1) / WPR;                 // of wavefront 0, the longest share
    if (mine <= 1) launch_wave_res<N, M, BITS, WPR, 1>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else if (mine <= 2) launch_wave_res<N, M, BITS, WPR, 2>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else if (mine <= 3) launch_wave_res<N, M, BITS, WPR, 3>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else if (mine <= 4) launch_wave_res<N, M, BITS, WPR, 4>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else launch_wave_res<N, M, BITS, WPR, MAXRES>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
}

template <int N, int M, int BITS>
void launch_wave(const float* W, int rows, int cols, int ldw, void* vals, void* meta, float* scales,
                 int vstride, int mstride, int flags, hipStream_t st)
{
    const int passes = (cols / M + 63) / 64;
    uint32_t* v = (uint32_t*)vals;
    uint32_t* m = (uint32_t*)meta;
    if (passes > 8) launch_wave_wpr<N, M, BITS, 4>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else if (passes > 4) launch_wave_wpr<N, M, BITS, 2>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
    else launch_wave_wpr<N, M, BITS, 1>(W, rows, cols, ldw, v, m, scales, vstride, mstride, flags, st);
}

}  // namespace

// Whether the wavefront-per-row kernels take a matrix: a compiled pattern, 16-byte aligned rows of
// W, dword-aligned outputs and packed rows that are whole dwords.
static bool wave_kernel_takes(const float* W, int cols, int ldw, int N, int M, int bits, const void* vals, const void* meta)
{
    const bool pattern_ok = (M == 4 && (N == 1 || N == 2 || N == 4)) || (M == 8 && (N == 1 || N == 2 || N == 4));
    const size_t kc = (size_t)cols / M * N;
    const int ib = index_bits(N, M);
    return pattern_ok && ((uintptr_t)W % 16 == 0) && (ldw % 4 == 0) && ((uintptr_t)vals % 4 == 0) &&
           ((uintptr_t)meta % 4 == 0) && (kc * bits % 32 == 0) && (kc * ib % 32 == 0);
}

int launch_compress(const float* W, int rows, int cols, int ldw, int N, int M, int bits, int layout, int rows_per_scale,
                    void* vals, void* meta, float* scales, hipStream_t st)
{
    const PackedArray pv = packed_values(cols, N, M, bits, layout), pm = packed_meta(cols, N, M, layout);
    const int vstride = (int)pv.stride, mstride = (int)pm.stride;
    bool done = false;
    begin_launch();
    // One scale per group of rows: the scales are computed first (row maxima, then the groups'),
    // and the kernels below quantise with what they find in scales[].
    // rows_per_scale 0: scales[] already holds the scales to use (the caller's own)
    const int given = rows_per_scale != 1 ? 1 : 0;
    const int flags = (given ? GIVEN_SCALES : 0) | (layout ? TILED_LAYOUT : 0);
    if (rows_per_scale > 1) launch_group_scales(W, rows, cols, ldw, rows_per_scale, (float)((1 << (bits - 1)) - 1), scales, st);
    if (wave_kernel_takes(W, cols, ldw, N, M, bits, vals, meta)) {
        done = true;
#define NM_CASE(n, m, b) else if (N == n && M == m && bits == b) launch_wave<n, m, b>(W, rows, cols, ldw, vals, meta, scales, vstride, mstride, flags, st)
        if (false) {}
        NM_CASE(2, 4, 8); NM_CASE(1, 4, 8); NM_CASE(2, 4, 4); NM_CASE(1, 4, 4); NM_CASE(4, 4, 8); NM_CASE(4, 4, 4);
        NM_CASE(1, 8, 8); NM_CASE(2, 8, 8); NM_CASE(4, 8, 8);
        NM_CASE(1, 8, 4); NM_CASE(2, 8, 4); NM_CASE(4, 8, 4);
        else done = false;
#undef NM_CASE
    }
    // the other patterns: a wavefront per row with the row's bits assembled in LDS
    const size_t image_bytes = 4 * (size_t)(vstride + mstride);       // four rows per workgroup
    if (!done && N < M && (uintptr_t)W % 16 == 0 && ldw % 4 == 0 && (uintptr_t)vals % 4 == 0 && (uintptr_t)meta % 4 == 0 &&
        vstride % 4 == 0 && mstride % 4 == 0 && image_bytes <= 64 * 1024) {
        const int rows_out = layout ? ((rows + 15) & ~15) : rows;
        done = true;
#define NM_CASE(n, m, b) else if (N == n && M == m && bits == b) \
        hipLaunchKernelGGL((compress_rowimage_kernel<n, m, b>), dim3((rows_out + 3) / 4), dim3(256), image_bytes, st, \
                           W, rows, cols, ldw, (uint8_t*)vals, (uint8_t*)meta, scales, pv, pm, given)
        if (false) {}
        NM_CASE(3, 4, 8); NM_CASE(3, 4, 4); NM_CASE(3, 8, 8); NM_CASE(3, 8, 4); NM_CASE(5, 8, 8); NM_CASE(5, 8, 4);
        NM_CASE(6, 8, 8); NM_CASE(6, 8, 4); NM_CASE(7, 8, 8); NM_CASE(7, 8, 4);
        else done = false;
#undef NM_CASE
    }
    if (!done) {
        const int rows_out = layout ? ((rows + 15) & ~15) : rows;
        hipLaunchKernelGGL(compress_generic_kernel, dim3((rows_out + 63) / 64), dim3(64), 0, st,
                           W, rows, cols, ldw, N, M, bits, (uint8_t*)vals, (uint8_t*)meta, scales, pv, pm, given);
    }
    return launch_status();
}

namespace {

int wave_wpr(int cols, int M)
{
    const int passes = (cols / M + 63) / 64;
    return passes > 8 ? 4 : (passes > 4 ? 2 : 1);
}

template <int N, int M, int BITS, bool ONCE>
void launch_batch_res(const BatchArgs& b, int max_mine, int blocks, hipStream_t st)
{
    constexpr int MAXRES = 16 / (M / 4);
    const dim3 grid((unsigned)blocks), wg(256);
    if (max_mine <= 1) hipLaunchKernelGGL((compress_batch_kernel<N, M, BITS, 1, ONCE>), grid, wg, 0, st, b);
    else if (max_mine <= 2) hipLaunchKernelGGL((compress_batch_kernel<N, M, BITS, 2, ONCE>), grid, wg, 0, st, b);
    else if (max_mine <= 3) hipLaunchKernelGGL((compress_batch_kernel<N, M, BITS, 3, ONCE>), grid, wg, 0, st, b);
    else if (max_mine <= 4) hipLaunchKernelGGL((compress_batch_kernel<N, M, BITS, 4, ONCE>), grid, wg, 0, st, b);
    else hipLaunchKernelGGL((compress_batch_kernel<N, M, BITS, MAXRES, ONCE>), grid, wg, 0, st, b);
}

template <int N, int M, int BITS>
void launch_batch(const BatchArgs& b, int max_mine, int blocks, hipStream_t st)
{
    if (b.stream_loads) launch_batch_res<N, M, BITS, true>(b, max_mine, blocks, st);
    else launch_batch_res<N, M, BITS, false>(b, max_mine, blocks, st);
}

}  // namespace

// Matrices that the wavefront kernel takes (alignment, whole dwords per packed row) go out in
// launches of up to BATCH_MAX; the others one by one through launch_compress.
int launch_compress_batch(const CompressItem* items, int count, int N, int M, int bits, int layout, hipStream_t st)
{
    begin_launch();
    BatchArgs b;
    b.count = 0;
    long long bytes = 0;
    for (int i = 0; i < count; ++i) bytes += (long long)items[i].rows * items[i].cols * 4;
    b.stream_loads = bytes > STREAM_ABOVE_BYTES ? 1 : 0;
    b.flags = layout ? TILED_LAYOUT : 0;
    int blocks = 0, max_mine = 0;
    auto flush = [&]() {
        if (b.count == 0) return;
#define NM_CASE(n, m, bt) else if (N == n && M == m && bits == bt) launch_batch<n, m, bt>(b, max_mine, blocks, st)
        if (false) {}
        NM_CASE(2, 4, 8); NM_CASE(1, 4, 8); NM_CASE(2, 4, 4); NM_CASE(1, 4, 4); NM_CASE(4, 4, 8); NM_CASE(4, 4, 4);
        NM_CASE(1, 8, 8); NM_CASE(2, 8, 8); NM_CASE(4, 8, 8);
        NM_CASE(1, 8, 4); NM_CASE(2, 8, 4); NM_CASE(4, 8, 4);
#undef NM_CASE
        b.count = 0; blocks = 0; max_mine = 0;
        for (int k = 0; k < BATCH_MAX; ++k) b.first_block[k] = 0x7FFFFFFF;
    };
    for (int k = 0; k < BATCH_MAX; ++k) b.first_block[k] = 0x7FFFFFFF;
    for (int i = 0; i < count; ++i) {
        const CompressItem& c = items[i];
        const PackedArray pv = packed_values(c.cols, N, M, bits, layout), pm = packed_meta(c.cols, N, M, layout);
        if (!wave_kernel_takes(c.W, c.cols, c.ldw, N, M, bits, c.vals, c.meta)) {
            int rc = launch_status();              // of the batches launched so far: the call below starts a bracket of its own
            if (rc == 0) rc = launch_compress(c.W, c.rows, c.cols, c.ldw, N, M, bits, layout, 1, c.vals, c.meta, c.scales, st);
            if (rc) return rc;
            continue;
        }
        const int wpr = wave_wpr(c.cols, M);
        const int passes = (c.cols / M + 63) / 64, mine = (passes + wpr - 1) / wpr, rpb = 4 / wpr;
        BatchItem& t = b.it[b.count++];
        t.W = c.W; t.vals = (uint32_t*)c.vals; t.meta = (uint32_t*)c.meta; t.scales = c.scales;
        t.rows = c.rows; t.cols = c.cols; t.ldw = c.ldw; t.vstride_dw = (int)pv.stride / 4; t.mstride_dw = (int)pm.stride / 4;
        t.wpr = wpr; t.first_block = blocks;
        b.first_block[b.count - 1] = blocks;
        const int rows_out = layout ? ((c.rows + 15) & ~15) : c.rows;     // the tiled layout pads the rows
        t.blocks = (rows_out + rpb - 1) / rpb;
        if (layout) t.blocks = (t.blocks + 7) & ~7;                       // whole rounds over the XCDs, see xcd_block
        blocks += t.blocks;
        max_mine = mine > max_mine ? mine : max_mine;
        if (b.count == BATCH_MAX) flush();
    }
    flush();
    return launch_status();
}

int launch_repack(const void* vals_in, const void* meta_in, int rows, int cols, int N, int M, int bits, int layout_in,
                  void* vals_out, void* meta_out, hipStream_t st)
{
    begin_launch();
    const int layout_out = 1 - layout_in;
    const int rows_out = layout_out ? ((rows + 15) & ~15) : rows;
    const PackedArray vs = packed_values(cols, N, M, bits, layout_in), vd = packed_values(cols, N, M, bits, layout_out);
    const PackedArray ms = packed_meta(cols, N, M, layout_in), md = packed_meta(cols, N, M, layout_out);
    const long long nv = (long long)rows_out * vs.stride, nmeta = (long long)rows_out * ms.stride;
    hipLaunchKernelGGL(repack_kernel, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t*)vals_in, (uint8_t*)vals_out, rows, rows_out, vs, vd);
    if (nmeta > 0)
        hipLaunchKernelGGL(repack_kernel, dim3((unsigned)((nmeta + 255) / 256)), dim3(256), 0, st,
                           (const uint8_t*)meta_in, (uint8_t*)meta_out, rows, rows_out, ms, md);
    return launch_status();
}

int launch_decompress(const void* vals, const void* meta, int rows, int cols, int N, int M, int bits, int layout,
                      int8_t* Wq, hipStream_t st)
{
    const long long total = (long long)rows * (cols / M);
    begin_launch();
    hipLaunchKernelGGL(decompress_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const uint8_t*)vals, (const uint8_t*)meta, rows, cols, N, M, bits,
                       packed_values(cols, N, M, bits, layout), packed_meta(cols, N, M, layout), Wq);
    return launch_status();
}

}  // namespace nm
