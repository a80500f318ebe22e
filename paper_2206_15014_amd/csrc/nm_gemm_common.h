// Device-side pieces shared by the nm_gemm kernels: MFMA operand types, the packed weight
// "unit" (load + decode to the sparse-MFMA operand form), and small helpers.
#ifndef NM_GEMM_COMMON_H
#define NM_GEMM_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace nm {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------------
// Weight units.  A unit is the slice of one packed weight row that covers 32 consecutive input
// columns: what one lane feeds to one sparse MFMA.
// ---------------------------------------------------------------------------------------------
// Four 4-bit two's-complement values, one in the low nibble of each byte (high nibbles zero), sign-
// extended to bytes: per byte (b ^ 8) - 8, done on the whole dword with the top bit of each byte
// set during the subtraction so that no borrow crosses a byte.
__device__ __forceinline__ uint32_t sext4x4(uint32_t nib)
{
    return ((nib ^ 0x88888888u) - 0x08080808u) ^ 0x80808080u;
}

template <int N, int M, int BITS>
struct Unit {
    static constexpr int IB = (M == 4) ? 2 : 4;
    static constexpr int EPU = 32 / M * N;          // kept entries per unit
    static constexpr int VBYTES = EPU * BITS / 8;   // packed value bytes per unit (2, 4, 8 or 16)
    static constexpr int MBYTES = EPU * IB / 8;     // packed index bytes per unit (2 or 4)
    static constexpr bool IDENTITY = (N == 2 && M == 4 && BITS == 8);

    struct Raw {
        uint32_t v[(VBYTES + 3) / 4];
        uint32_t m;
    };

    static __device__ __forceinline__ Raw load(const uint8_t* __restrict__ vrow, const uint8_t* __restrict__ mrow, int unit)
    {
        Raw r;
        const uint8_t* pv = vrow + (size_t)unit * VBYTES;
        if constexpr (VBYTES == 16) {
            uint4 t = *reinterpret_cast<const uint4*>(pv);
            r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
        } else if constexpr (VBYTES == 8) {
            uint2 t = *reinterpret_cast<const uint2*>(pv);
            r.v[0] = t.x; r.v[1] = t.y;
        } else if constexpr (VBYTES == 4) {
            r.v[0] = *reinterpret_cast<const uint32_t*>(pv);
        } else {
            r.v[0] = *reinterpret_cast<const uint16_t*>(pv);
        }
        const uint8_t* pm = mrow + (size_t)unit * MBYTES;
        if constexpr (MBYTES == 4) r.m = *reinterpret_cast<const uint32_t*>(pm);
        else r.m = *reinterpret_cast<const uint16_t*>(pm);
        return r;
    }

    // Packed unit -> MFMA operand: 16 int8 codes (zero where nothing is kept) and 16 2-bit positions.
    static __device__ __forceinline__ void decode(const Raw& r, v4i& codes, int& pos)
    {
        if constexpr (IDENTITY) {
            codes = v4i{(int)r.v[0], (int)r.v[1], (int)r.v[2], (int)r.v[3]};
            pos = (int)r.m;
        } else if constexpr (M == 4) {
            // Whole dwords at a time (the per-entry form below costs ~6 vector-ALU operations per
            // kept entry, several times the MFMA time of the fragment).  Operand byte 2g+j is slot
            // j of group g; a pattern that keeps one entry per group fills slot 0 and leaves slot 1
            // zero, whose position bits may then be anything.
            uint32_t w[EPU / 4];                               // the codes as bytes, in entry order
            if constexpr (BITS == 8) {
#pragma unroll
                for (int d = 0; d < EPU / 4; ++d) w[d] = r.v[d];
            } else {
#pragma unroll
                for (int d = 0; d < EPU / 8; ++d) {
                    const uint32_t x = r.v[d];
                    const uint32_t lo = sext4x4(x & 0x0F0F0F0Fu);          // entries 0, 2, 4, 6 of this dword
                    const uint32_t hi = sext4x4((x >> 4) & 0x0F0F0F0Fu);   // entries 1, 3, 5, 7
                    w[2 * d] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                    w[2 * d + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
                }
            }
            if constexpr (N == 2) {
                codes = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
                pos = (int)r.m;
            } else {
                // entry i -> byte 2i, zero in byte 2i+1; its 2 position bits -> bits 4i, 4i+1
                codes = v4i{(int)__builtin_amdgcn_perm(0u, w[0], 0x0c010c00u), (int)__builtin_amdgcn_perm(0u, w[0], 0x0c030c02u),
                            (int)__builtin_amdgcn_perm(0u, w[1], 0x0c010c00u), (int)__builtin_amdgcn_perm(0u, w[1], 0x0c030c02u)};
                uint32_t x = r.m & 0xFFFFu;
                x = (x | (x << 8)) & 0x00FF00FFu;
                x = (x | (x << 4)) & 0x0F0F0F0Fu;
                x = (x | (x << 2)) & 0x33333333u;
                pos = (int)x;
            }
        } else if constexpr (M == 8 && N <= 2) {
            // A group of 8 columns is two operand groups of 4 ("halves").  Kept entry j of a group
            // goes to slot j of the half its column lies in (bit 2 of its offset); the other slots
            // hold zero.  All four groups of the unit are handled at once, one byte lane per group.
            uint32_t w[2];                                     // the codes as bytes, in entry order
            if constexpr (BITS == 8) {
                w[0] = r.v[0];
                if constexpr (N == 2) w[1] = r.v[1];
                else w[1] = 0u;
            } else {
                const uint32_t x = r.v[0];
                const uint32_t lo = sext4x4(x & 0x0F0F0F0Fu);
                const uint32_t hi = sext4x4((x >> 4) & 0x0F0F0F0Fu);
                w[0] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                w[1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
            }
            if constexpr (N == 2) {
                const uint32_t m = r.m;                        // byte g = offset a | offset b << 4 of group g
                const uint32_t ma = ((m >> 2) & 0x01010101u) * 255u;   // 0xFF where a lies in the upper half
                const uint32_t mb = ((m >> 6) & 0x01010101u) * 255u;
                const uint32_t a3 = m & 0x03030303u, b3 = (m >> 4) & 0x03030303u;
                pos = (int)((((a3 << 4) & ma) | (a3 & ~ma)) | (((b3 << 6) & mb) | ((b3 << 2) & ~mb)));
                // group g: (qa, qb, qa, qb) masked with (~ma, ~mb, ma, mb) of that group
                const uint32_t k0 = __builtin_amdgcn_perm(mb, ma, 0x04000400u) ^ 0x0000FFFFu;
                const uint32_t k1 = __builtin_amdgcn_perm(mb, ma, 0x05010501u) ^ 0x0000FFFFu;
                const uint32_t k2 = __builtin_amdgcn_perm(mb, ma, 0x06020602u) ^ 0x0000FFFFu;
                const uint32_t k3 = __builtin_amdgcn_perm(mb, ma, 0x07030703u) ^ 0x0000FFFFu;
                codes = v4i{(int)(__builtin_amdgcn_perm(0u, w[0], 0x01000100u) & k0),
                            (int)(__builtin_amdgcn_perm(0u, w[0], 0x03020302u) & k1),
                            (int)(__builtin_amdgcn_perm(0u, w[1], 0x01000100u) & k2),
                            (int)(__builtin_amdgcn_perm(0u, w[1], 0x03020302u) & k3)};
            } else {
                uint32_t y = r.m & 0xFFFFu;                    // four 4-bit offsets -> one per byte
                y = (y | (y << 8)) & 0x00FF00FFu;
                y = (y | (y << 4)) & 0x0F0F0F0Fu;
                const uint32_t ma = ((y >> 2) & 0x01010101u) * 255u;
                const uint32_t a3 = y & 0x03030303u;
                pos = (int)(((a3 << 4) & ma) | (a3 & ~ma));
                // group g: (q, 0, q, 0) masked with (~ma, 0, ma, 0) of that group
                codes = v4i{(int)(__builtin_amdgcn_perm(0u, w[0], 0x0c000c00u) & (__builtin_amdgcn_perm(0u, ma, 0x0c000c00u) ^ 0x000000FFu)),
                            (int)(__builtin_amdgcn_perm(0u, w[0], 0x0c010c01u) & (__builtin_amdgcn_perm(0u, ma, 0x0c010c01u) ^ 0x000000FFu)),
                            (int)(__builtin_amdgcn_perm(0u, w[0], 0x0c020c02u) & (__builtin_amdgcn_perm(0u, ma, 0x0c020c02u) ^ 0x000000FFu)),
                            (int)(__builtin_amdgcn_perm(0u, w[0], 0x0c030c03u) & (__builtin_amdgcn_perm(0u, ma, 0x0c030c03u) ^ 0x000000FFu))};
            }
        } else {
            uint32_t hv[4] = {0u, 0u, 0u, 0u};
            uint32_t hp = 0u;
#pragma unroll
            for (int e = 0; e < EPU; ++e) {
                uint32_t q;
                if constexpr (BITS == 8) {
                    q = (r.v[e / 4] >> (8 * (e % 4))) & 0xFFu;
                } else {
                    uint32_t nib = (r.v[e / 8] >> (4 * (e % 8))) & 0xFu;
                    q = ((nib ^ 8u) - 8u) & 0xFFu;                 // sign-extend 4 -> 8 bits
                }
                const uint32_t off = (r.m >> (e * IB)) & (uint32_t)(M - 1);
                const int g = e / N, j = e % N;                    // group inside the unit, rank inside the group
                if constexpr (M == 4) {
                    const int he = 2 * g + j;                      // slot j of subgroup g
                    hv[he / 4] |= q << (8 * (he % 4));
                    hp |= off << (2 * he);
                } else {
                    const uint32_t byte = 2u * (off >> 2) + (uint32_t)j;   // subgroup 2g + off/4, slot j
                    hv[g] |= q << (8u * byte);
                    hp |= (off & 3u) << (2u * (4u * (uint32_t)g + byte));
                }
            }
            codes = v4i{(int)hv[0], (int)hv[1], (int)hv[2], (int)hv[3]};
            pos = (int)hp;
        }
    }
};

// ---------------------------------------------------------------------------------------------
// LDS-direct operand staging (global_load_lds_dwordx4): geometry of one ring stage and the load /
// wait primitives.  A direct load writes 64 lanes x 16 bytes to 1 KB of consecutive LDS in lane
// order, so every staged array is a sequence of 1 KB blocks and the layout inside a block is
// chosen by which global chunk each lane fetches.
// ---------------------------------------------------------------------------------------------
template <int N, int M, int BITS, int BT, int BO, int KU>
struct DmaGeom {
    using U = Unit<N, M, BITS>;
    static constexpr int RVS = 4 * U::VBYTES * KU;           // packed value bytes per row per stage, in memory
    static constexpr int RMS = 4 * U::MBYTES * KU;           // packed index bytes per row per stage, in memory
    // A direct load moves 16-byte pieces.  An array with only 8 bytes per row and stage is staged
    // as the 16-byte piece that holds two consecutive stages ("pair"): every stage loads the piece
    // its K block lies in and reads its own half.
    static constexpr bool PAIR_V = (RVS == 8), PAIR_M = (RMS == 8);
    static constexpr int RV = PAIR_V ? 16 : RVS;             // bytes per row in the LDS stage
    static constexpr int RM = PAIR_M ? 16 : RMS;
    static_assert(RV % 16 == 0 && RM % 16 == 0, "rows must be whole 16-byte chunks");
    static constexpr bool V_SWIZZLE = (RV == 128);           // 8 chunks per row: same XOR as the X rows
    // XOR term for the 16-byte chunk index of a codes row, so that the 16 rows one fragment read
    // touches spread over all banks: rows 256 bytes apart would otherwise meet in the same banks
    // (every 2nd row of 128 bytes, every 4th of 64, every 8th of 32).
    __host__ __device__ static constexpr int v_xor(int row)
    {
        return RV == 128 ? ((row >> 1) & 7) : RV == 64 ? ((row >> 2) & 3) : RV == 32 ? ((row >> 3) & 1) : 0;
    }
    static constexpr int X_SUB = BT * 128;                   // bytes of one 128-column slice of X
    static constexpr int X_BLOCKS = KU * BT * 128 / 1024;
    static constexpr int V_BLOCKS = (BO * RV + 1023) / 1024;
    static constexpr int M_BLOCKS = (BO * RM + 1023) / 1024;
    static constexpr int X_OFF = 0;
    static constexpr int V_OFF = X_BLOCKS * 1024;
    static constexpr int M_OFF = V_OFF + V_BLOCKS * 1024;
    static constexpr int BLOCKS = X_BLOCKS + V_BLOCKS + M_BLOCKS;
};

// One direct-to-LDS load: 64 lanes x 16 bytes, lane l from its own pointer to LDS lds_addr + 16*l.
// (M0 carries the LDS address, which must be the same in every lane; one wait state between
// writing M0 and the load that reads it.)
__device__ __forceinline__ void dma16(uint32_t lds_addr, const uint8_t* src)
{
    lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(src)
                 : "memory");
}

// The same with the address split into a scalar base and a 32-bit per-lane byte offset (no 64-bit
// vector arithmetic to form it).  `base` must be the same in every lane.
__device__ __forceinline__ void dma16s(uint32_t lds_addr, uint32_t offset, const uint8_t* base)
{
    lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
    const uint64_t b = (uint64_t)(uintptr_t)base;
    const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(offset), "s"(sb)
                 : "memory");
}

// 16-byte store at agent scope: the line is written through to memory as it is stored instead of
// staying dirty in this XCD's L2 until the end-of-kernel write-back, which for outputs larger
// than the L2s hold would otherwise stand between this kernel's last wavefront and the next
// kernel's first.  (The compiler does not see the instruction, hence the wait state that a wide
// store needs before its data registers may be overwritten.)
__device__ __forceinline__ void store16_through(void* dst, v4i v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
}

template <int CNT>
__device__ __forceinline__ void wait_vm()
{
    static_assert(CNT >= 0 && CNT < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(CNT) : "memory");
}

// Compile-time counted loop: f(std::integral_constant<int, 0>{}) ... f(std::integral_constant<int, COUNT-1>{}).
template <int COUNT, class F, int I = 0>
__device__ __forceinline__ void int_for(F&& f)
{
    if constexpr (I < COUNT) {
        f(std::integral_constant<int, I>{});
        int_for<COUNT, F, I + 1>(static_cast<F&&>(f));
    }
}

// Two fp32 -> two bf16 (round to nearest even) in one dword, `lo` in bits 0..15: gfx950 converts
// a pair per instruction (v_cvt_pk_bf16_f32), which matters because the epilogue's vector ALU
// work per output is of the same order as the matrix-pipe work per output at K = 768.
typedef __bf16 nm_bf16x2 __attribute__((ext_vector_type(2)));
typedef float nm_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const nm_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, nm_bf16x2));
}

// Requantised output (Eq. 4, then Eq. 5 at 8 bits, both with offset 0), as the declaration of
// nm_gemm_q8 fixes it: per column g = (act_scale * scale) / out_scale and h = bias / out_scale (one
// fp32 operation each, true divisions), per output z = fma(float(acc), g, h) and
// code = clamp(rne(z), -127, 127).
__device__ __forceinline__ void requant_column(float act_scale, float scale, float bias, float out_scale, float& g, float& h)
{
    g = __fdiv_rn(act_scale * scale, out_scale);
    h = __fdiv_rn(bias, out_scale);
}

// The four outputs a lane holds of one token, as four codes packed little-endian (column r in
// byte r); `m` collects max |z|.
__device__ __forceinline__ uint32_t requant4(const v4i c, const float (&g)[4], const float (&h)[4], float& m)
{
    // clamp(rne(z)) = rne(clamp(z)) because the bounds are integers; adding 1.5 * 2^23 to a value of
    // magnitude <= 127 rounds it to an integer (nearest, ties to even: the add's own rounding) and
    // leaves that integer, in two's complement, in the low byte of the sum's bit pattern.
    uint32_t t[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float z = __fmaf_rn((float)c[r], g[r], h[r]);
        m = fmaxf(m, fabsf(z));
        t[r] = __float_as_uint(__builtin_amdgcn_fmed3f(z, -127.0f, 127.0f) + 12582912.0f);
    }
    // bytes 0 of t[0..3] -> one dword
    const uint32_t lo = __builtin_amdgcn_perm(t[1], t[0], 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(t[3], t[2], 0x04000c0cu);
    return lo | hi;
}

// Largest of `m` (>= 0) over the wavefront, max-combined into *dst: non-negative floats order like
// their bit patterns, so an unsigned atomic maximum does it.  Thousands of wavefronts meet at that
// one address and an atomic there costs some 15 ns, so a wavefront first reads the value (at agent
// scope; it only ever grows, so one that is too old merely costs an atomic that was not needed)
// and leaves the atomic out unless its own is larger - which after the first few is rare.
// Every lane of the wavefront must call it.  `m` is in units of the codes: the value committed is
// m * out_scale (multiplying by a positive number keeps the order, so the largest product is the
// product of the largest).
__device__ __forceinline__ void absmax_commit(float m, float out_scale, float* dst)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    m = m * out_scale;
    if ((threadIdx.x & 63) == 0 && dst != nullptr) {
        unsigned int* u = reinterpret_cast<unsigned int*>(dst);
        if (__float_as_uint(m) > __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(u, __float_as_uint(m));
    }
}

// Epilogue shared by the MFMA kernels: Eq. 4 with offset 0 applied to the product of two quantised
// operands.  acc[fo][ft] is the 16x16 accumulator fragment of weight rows o_base + fo*16 .. and
// tokens t_base + ft*16 ..; lane (li, lg) holds rows 4*lg .. 4*lg+3 of token li.
template <int FO, int FT, class Args>
__device__ __forceinline__ void store_tile(const Args& a, const v4i (&acc)[FO][FT], int o_base, int t_base, int li, int lg)
{
    float m = 0.0f;                            // max |y| of this lane (requantised output only)
#pragma unroll
    for (int fo = 0; fo < FO; ++fo) {
        const int o = o_base + fo * 16 + 4 * lg;
        if (o >= a.O) continue;
        const float4 sw = *reinterpret_cast<const float4*>(a.scales + o);
        const float sws[4] = {sw.x, sw.y, sw.z, sw.w};
        const float sc[4] = {a.act_scale * sw.x, a.act_scale * sw.y, a.act_scale * sw.z, a.act_scale * sw.w};
        float bs[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.bias) {
            const float4 b = *reinterpret_cast<const float4*>(a.bias + o);
            bs[0] = b.x; bs[1] = b.y; bs[2] = b.z; bs[3] = b.w;
        }
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const int t = t_base + ft * 16 + li;
            if (t >= a.tokens) continue;
            const v4i c = acc[fo][ft];
            const size_t at = (size_t)t * a.ldo + o;
            if (a.acc) *reinterpret_cast<v4i*>(a.acc + at) = c;
            if (a.out_dtype != 0) {
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = (float)c[r] * sc[r] + bs[r];
                if (a.out_dtype == 1) {
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + at) = make_float4(y[0], y[1], y[2], y[3]);
                } else if (a.out_dtype == 2) {
                    uint2 p;
                    p.x = pack_bf16x2(y[0], y[1]);
                    p.y = pack_bf16x2(y[2], y[3]);
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + at) = p;
                } else {
                    float g[4], h[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) requant_column(a.act_scale, sws[r], bs[r], a.out_scale, g[r], h[r]);
                    *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.out) + at) = requant4(c, g, h, m);
                }
            }
        }
    }
    if (a.out_dtype == 3) absmax_commit(m, a.out_scale, a.absmax);
}

// Same, with the row scales and biases already in registers (sw[fo], bw[fo] hold rows
// o_base + fo*16 + 4*lg .. +3).  For requantised output (out_dtype 3) they hold the columns'
// multipliers g and offsets h instead.
template <int FO, int FT, class Args>
__device__ __forceinline__ void store_tile_pre(const Args& a, const v4i (&acc)[FO][FT], const float4 (&sw)[FO], const float4 (&bw)[FO],
                                               int o_base, int t_base, int li, int lg)
{
    float m = 0.0f;                            // max |y| of this lane (requantised output only)
#pragma unroll
    for (int fo = 0; fo < FO; ++fo) {
        const int o = o_base + fo * 16 + 4 * lg;
        if (o >= a.O) continue;
        const float sc[4] = {a.act_scale * sw[fo].x, a.act_scale * sw[fo].y, a.act_scale * sw[fo].z, a.act_scale * sw[fo].w};
        const float bs[4] = {bw[fo].x, bw[fo].y, bw[fo].z, bw[fo].w};
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const int t = t_base + ft * 16 + li;
            if (t >= a.tokens) continue;
            const v4i c = acc[fo][ft];
            const size_t at = (size_t)t * a.ldo + o;
            if (a.acc) *reinterpret_cast<v4i*>(a.acc + at) = c;
            if (a.out_dtype != 0) {
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = (float)c[r] * sc[r] + bs[r];
                if (a.out_dtype == 1) {
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + at) = make_float4(y[0], y[1], y[2], y[3]);
                } else if (a.out_dtype == 2) {
                    uint2 p;
                    p.x = pack_bf16x2(y[0], y[1]);
                    p.y = pack_bf16x2(y[2], y[3]);
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + at) = p;
                } else {
                    const float g[4] = {sw[fo].x, sw[fo].y, sw[fo].z, sw[fo].w};
                    *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.out) + at) = requant4(c, g, bs, m);
                }
            }
        }
    }
    if (a.out_dtype == 3) absmax_commit(m, a.out_scale, a.absmax);
}

}  // namespace
}  // namespace nm

#endif
