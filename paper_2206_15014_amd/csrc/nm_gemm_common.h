// Device-side pieces shared by the nm_gemm kernels: MFMA operand types, the packed weight
// "unit" (load + decode to the sparse-MFMA operand form), and small helpers.
#ifndef NM_GEMM_COMMON_H
#define NM_GEMM_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "nm_internal.h"

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
    static constexpr int IB = (N >= M) ? 0 : (M == 4) ? 2 : 4;
    static constexpr int EPU = 32 / M * N;          // kept entries per unit
    static constexpr int VBYTES = EPU * BITS / 8;   // packed value bytes per unit (2 .. 32)
    static constexpr int MBYTES = EPU * IB / 8;     // packed index bytes per unit (0 for a dense matrix)
    static constexpr bool IDENTITY = (N == 2 && M == 4 && BITS == 8);
    // More than two kept entries can fall into one aligned subgroup of four columns: the unit is
    // then split into two legal operands of the sparse MFMA (see decode2).
    static constexpr bool DUAL = (N > 2);
    static constexpr int VD = (VBYTES + 3) / 4, MD = (MBYTES + 3) / 4 > 0 ? (MBYTES + 3) / 4 : 1;

    struct Raw {
        uint32_t v[VD];
        uint32_t m[MD];
    };

    // Row layout: unit `unit` of the packed row at vrow / mrow (patterns with whole power-of-two units).
    static __device__ __forceinline__ Raw load(const uint8_t* __restrict__ vrow, const uint8_t* __restrict__ mrow, int unit)
    {
        static_assert(!DUAL, "row-layout loads serve the patterns with at most two kept per group");
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
        if constexpr (MBYTES == 4) r.m[0] = *reinterpret_cast<const uint32_t*>(pm);
        else r.m[0] = *reinterpret_cast<const uint16_t*>(pm);
        return r;
    }

    // Tiled layout: `vblock` / `mblock` point at the block (16 rows x 128 columns) in LDS, `lane`
    // = 16 * (unit of the slice) + (row of the block) is this lane's unit.  Piece p of a unit of
    // UB bytes lies at (p * 64 + lane) * PB: every read is lane-contiguous, free of bank conflicts.
    template <int UB, int WORDS>
    static __device__ __forceinline__ void load_pieces(const uint8_t* __restrict__ block, int lane, uint32_t (&dst)[WORDS])
    {
        constexpr int PB = piece_bytes(UB), P = UB / PB;
#pragma unroll
        for (int w = 0; w < WORDS; ++w) dst[w] = 0u;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const uint8_t* q = block + (p * 64 + lane) * PB;
            if constexpr (PB == 16) {
                const uint4 t = *reinterpret_cast<const uint4*>(q);
                dst[4 * p] = t.x; dst[4 * p + 1] = t.y; dst[4 * p + 2] = t.z; dst[4 * p + 3] = t.w;
            } else if constexpr (PB == 8) {
                const uint2 t = *reinterpret_cast<const uint2*>(q);
                dst[2 * p] = t.x; dst[2 * p + 1] = t.y;
            } else if constexpr (PB == 4) {
                dst[p] = *reinterpret_cast<const uint32_t*>(q);
            } else {
                static_assert(PB == 2, "units are an even number of bytes");
                dst[p / 2] |= (uint32_t)*reinterpret_cast<const uint16_t*>(q) << (16 * (p & 1));
            }
        }
    }
    static __device__ __forceinline__ Raw load_tiled(const uint8_t* __restrict__ vblock, const uint8_t* __restrict__ mblock, int lane)
    {
        Raw r;
        load_pieces<VBYTES>(vblock, lane, r.v);
        if constexpr (MBYTES > 0) load_pieces<MBYTES>(mblock, lane, r.m);
        else r.m[0] = 0u;
        return r;
    }

    // Packed unit -> MFMA operand: 16 int8 codes (zero where nothing is kept) and 16 2-bit positions.
    static __device__ __forceinline__ void decode(const Raw& r_in, v4i& codes, int& pos)
    {
        static_assert(!DUAL, "one operand holds at most two entries per subgroup of four");
        struct { const uint32_t* v; uint32_t m; } r = {r_in.v, r_in.m[0]};
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

    // Patterns that can keep more than two entries in an aligned subgroup of four columns (3:4,
    // 3:8 .. 7:8, dense): the unit becomes TWO legal operands of the sparse MFMA, multiplied one after the
    // other against the same activations.  Of the (up to four) entries a subgroup keeps, operand
    // 1 takes the first two and operand 2 the rest, zero where there is none.  The sparse
    // instruction at twice its issue count does the work of the dense one at the same rate, and
    // the whole staging path stays as it is.
    static __device__ __forceinline__ void decode2(const Raw& r, v4i& c1, int& p1, v4i& c2, int& p2)
    {
        static_assert(DUAL, "patterns with more than two kept entries per group");
        // the codes as bytes, in entry order (4-bit units may end in the middle of a dword)
        uint32_t w[2 * ((EPU + 7) / 8)];
        if constexpr (BITS == 8) {
#pragma unroll
            for (int d = 0; d < EPU / 4; ++d) w[d] = r.v[d];
        } else {
#pragma unroll
            for (int d = 0; d < (EPU + 7) / 8; ++d) {
                const uint32_t x = r.v[d];
                const uint32_t lo = sext4x4(x & 0x0F0F0F0Fu);          // entries 0, 2, 4, 6 of this dword
                const uint32_t hi = sext4x4((x >> 4) & 0x0F0F0F0Fu);   // entries 1, 3, 5, 7
                w[2 * d] = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                w[2 * d + 1] = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
            }
        }
        if constexpr (N == M) {
            // dense: dword d of w is subgroup d (columns 4d .. 4d+3); operand dword h covers subgroups
            // 2h and 2h+1: columns 0, 1 of each go to operand 1 (positions 0, 1), columns 2, 3 to operand 2
            c1 = v4i{(int)__builtin_amdgcn_perm(w[1], w[0], 0x05040100u), (int)__builtin_amdgcn_perm(w[3], w[2], 0x05040100u),
                     (int)__builtin_amdgcn_perm(w[5], w[4], 0x05040100u), (int)__builtin_amdgcn_perm(w[7], w[6], 0x05040100u)};
            c2 = v4i{(int)__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), (int)__builtin_amdgcn_perm(w[3], w[2], 0x07060302u),
                     (int)__builtin_amdgcn_perm(w[5], w[4], 0x07060302u), (int)__builtin_amdgcn_perm(w[7], w[6], 0x07060302u)};
            p1 = 0x44444444;                                   // slot 0 at position 0, slot 1 at position 1
            p2 = (int)0xEEEEEEEEu;                             // slot 0 at position 2, slot 1 at position 3
        } else if constexpr (N == 3 && M == 4) {
            // subgroup g keeps entries 3g, 3g+1, 3g+2: the first two to operand 1, the third to slot 0
            // of operand 2, whose slot 1 is zero.  Operand dword h = subgroups 2h, 2h+1 = bytes 6h ...
            c1 = v4i{(int)__builtin_amdgcn_perm(w[1], w[0], 0x04030100u), (int)__builtin_amdgcn_perm(w[2], w[1], 0x06050302u),
                     (int)__builtin_amdgcn_perm(w[4], w[3], 0x04030100u), (int)__builtin_amdgcn_perm(w[5], w[4], 0x06050302u)};
            c2 = v4i{(int)__builtin_amdgcn_perm(w[1], w[0], 0x0c050c02u), (int)__builtin_amdgcn_perm(w[2], w[1], 0x0c070c04u),
                     (int)__builtin_amdgcn_perm(w[4], w[3], 0x0c050c02u), (int)__builtin_amdgcn_perm(w[5], w[4], 0x0c070c04u)};
            // index bits: 6 per subgroup (o0 | o1 << 2 | o2 << 4), 48 in all
            const uint64_t m = (uint64_t)r.m[0] | ((uint64_t)r.m[1] << 32);
            uint32_t q1 = 0u, q2 = 0u;
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                q1 |= (uint32_t)((m >> (6 * g)) & 0xFu) << (4 * g);
                q2 |= (uint32_t)((m >> (6 * g + 4)) & 0x3u) << (4 * g);
            }
            p1 = (int)q1;
            p2 = (int)(q2 | 0xCCCCCCCCu);                      // the empty slot points at column 3 (its code is zero)
        } else {
            static_assert(M == 8 && N >= 3 && N < 8, "dual operands: 3:4, 3:8 .. 7:8 and dense");
            // group g (8 columns) keeps entries N*g .. N*g+N-1 of the unit, one byte of w and one
            // 4-bit offset each: the codes are scattered to their columns (zeros elsewhere) and the
            // 8 columns then split as a dense group
            uint32_t a1[4], a2[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint64_t d = 0;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    const int e = N * g + j;
                    const uint32_t code = (w[e / 4] >> (8 * (e % 4))) & 0xFFu;
                    const uint32_t sh = ((r.m[e / 8] >> (4 * (e % 8))) & 7u) * 8u;
                    d |= (uint64_t)code << sh;
                }
                const uint32_t lo = (uint32_t)d, hi = (uint32_t)(d >> 32);
                a1[g] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                a2[g] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
            }
            c1 = v4i{(int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
            c2 = v4i{(int)a2[0], (int)a2[1], (int)a2[2], (int)a2[3]};
            p1 = 0x44444444;
            p2 = (int)0xEEEEEEEEu;
        }
    }
};

// ---------------------------------------------------------------------------------------------
// LDS-direct operand staging (global_load_lds_dwordx4): geometry of one ring stage and the load /
// wait primitives.  A direct load writes 64 lanes x 16 bytes to 1 KB of consecutive LDS in lane
// order, so every staged array is a sequence of 1 KB blocks and the layout inside a block is
// chosen by which global chunk each lane fetches.  The packed weights are staged as copies of the
// tiled layout's blocks (16 rows x 128 columns each): [slice of the stage][row block of the tile].
// ---------------------------------------------------------------------------------------------
template <int N, int M, int BITS, int BT, int BO, int KU>
struct DmaGeom {
    using U = Unit<N, M, BITS>;
    static constexpr int FB = BO / 16;                       // row blocks (weight fragments) per tile
    static constexpr int VBLK = 64 * U::VBYTES;              // bytes of one block of the tiled layout: codes ...
    static constexpr int MBLK = 64 * U::MBYTES;              // ... and index bits (0: dense matrix)
    static constexpr int MBLK_ = MBLK > 0 ? MBLK : 1;        // as a divisor
    static constexpr int V_BYTES = KU * FB * VBLK;           // per stage
    static constexpr int M_BYTES = KU * FB * MBLK;
    static_assert(VBLK % 16 == 0 && MBLK % 16 == 0, "blocks are whole 16-byte pieces");
    static constexpr int X_SUB = BT * 128;                   // bytes of one 128-column slice of X
    static constexpr int X_BLOCKS = KU * BT * 128 / 1024;
    static constexpr int V_BLOCKS = (V_BYTES + 1023) / 1024;
    static constexpr int M_BLOCKS = (M_BYTES + 1023) / 1024;
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

// 16-byte store at system scope: the line is written through to memory as it is stored instead of
// staying dirty in this XCD's L2 until the end-of-kernel write-back, which for outputs larger
// than the L2s hold would otherwise stand between this kernel's last wavefront and the next
// kernel's first.  (Measured on 19 to 100 MB of bf16: agent scope, sc1 alone, takes 1 to 3 %
// longer; the default and sc0 alone 20 %; the non-temporal hint helps none of them.  The
// compiler does not see the instruction, hence the wait state that a wide store needs before its
// data registers may be overwritten.)
__device__ __forceinline__ void store16_through(void* dst, v4i v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
}

typedef int v2i_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store8_through(void* dst, v2i_t v)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
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
    // in-register lane moves (DPP within rows of 16, then across the rows): lane 63 ends up with the
    // maximum of all 64; six round trips through the LDS crossbar cost a microsecond of latency
#define NM_MAX_STEP(ctrl, row_mask) \
    m = fmaxf(m, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(m), ctrl, row_mask, 0xF, false)))
    NM_MAX_STEP(0x111, 0xF);   // row_shr:1
    NM_MAX_STEP(0x112, 0xF);   // row_shr:2
    NM_MAX_STEP(0x114, 0xF);   // row_shr:4
    NM_MAX_STEP(0x118, 0xF);   // row_shr:8
    NM_MAX_STEP(0x142, 0xA);   // row_bcast:15 -> rows 1 and 3
    NM_MAX_STEP(0x143, 0xC);   // row_bcast:31 -> rows 2 and 3
#undef NM_MAX_STEP
    m = m * out_scale;
    if ((threadIdx.x & 63) == 63 && dst != nullptr) {
        unsigned int* u = reinterpret_cast<unsigned int*>(dst);
        if (__float_as_uint(m) > __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(u, __float_as_uint(m));
    }
}

// The activation scale and the scale of the output codes: the host value, or the device float that
// replaces it (a scale that earlier work on the stream has computed).
template <class Args>
__device__ __forceinline__ float act_scale_of(const Args& a)
{
    return a.act_scale_dev ? *a.act_scale_dev : a.act_scale;
}
template <class Args>
__device__ __forceinline__ float out_scale_of(const Args& a)
{
    return a.out_scale_dev ? *a.out_scale_dev : a.out_scale;
}

// Epilogue shared by the MFMA kernels: Eq. 4 with offset 0 applied to the product of two quantised
// operands.  acc[fo][ft] is the 16x16 accumulator fragment of weight rows o_base + fo*16 .. and
// tokens t_base + ft*16 ..; lane (li, lg) holds rows 4*lg .. 4*lg+3 of token li.
template <int FO, int FT, class Args>
__device__ __forceinline__ void store_tile(const Args& a, const v4i (&acc)[FO][FT], int o_base, int t_base, int li, int lg)
{
    float m = 0.0f;                            // max |y| of this lane (requantised output only)
    const float s_act = act_scale_of(a), s_out = out_scale_of(a);
#pragma unroll
    for (int fo = 0; fo < FO; ++fo) {
        const int o = o_base + fo * 16 + 4 * lg;
        if (o >= a.O) continue;
        const float4 sw = *reinterpret_cast<const float4*>(a.scales + o);
        const float sws[4] = {sw.x, sw.y, sw.z, sw.w};
        const float sc[4] = {s_act * sw.x, s_act * sw.y, s_act * sw.z, s_act * sw.w};
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
                    for (int r = 0; r < 4; ++r) requant_column(s_act, sws[r], bs[r], s_out, g[r], h[r]);
                    *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.out) + at) = requant4(c, g, h, m);
                }
            }
        }
    }
    if (a.out_dtype == 3) absmax_commit(m, s_out, a.absmax);
}

// Same, with the row scales and biases already in registers (sw[fo], bw[fo] hold rows
// o_base + fo*16 + 4*lg .. +3).  For requantised output (out_dtype 3) they hold the columns'
// multipliers g and offsets h instead.
template <int FO, int FT, class Args>
__device__ __forceinline__ void store_tile_pre(const Args& a, const v4i (&acc)[FO][FT], const float4 (&sw)[FO], const float4 (&bw)[FO],
                                               int o_base, int t_base, int li, int lg)
{
    float m = 0.0f;                            // max |y| of this lane (requantised output only)
    const float s_act = act_scale_of(a);
#pragma unroll
    for (int fo = 0; fo < FO; ++fo) {
        const int o = o_base + fo * 16 + 4 * lg;
        if (o >= a.O) continue;
        const float sc[4] = {s_act * sw[fo].x, s_act * sw[fo].y, s_act * sw[fo].z, s_act * sw[fo].w};
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
    if (a.out_dtype == 3) absmax_commit(m, out_scale_of(a), a.absmax);
}

}  // namespace
}  // namespace nm

#endif
