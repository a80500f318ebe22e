// nm_gemm, LDS-direct variant for gfx950: operands go global -> LDS with
// global_load_lds_dwordx4 (no register staging, no LDS store instructions), through a ring of
// STAGES stages, and the sparse MFMA reads its fragments from there.
//
// Why: at these layer shapes one workgroup per CU streams its X tile (first touch from HBM,
// about a microsecond away) and its slice of the packed weights (from L2) at the CU's L1 fill
// rate; that, the LDS traffic of the fragment reads and - in a K loop that keeps every CU busy
// for long - the board's power limit (the clock is pulled down) bound the loop, not the MFMA
// pipe.  Keeping several stages of loads in flight without spending registers or LDS-store
// issue slots is what the direct-to-LDS load is for; the packed weight bytes travel in their
// compact form and are widened / re-encoded to the MFMA operand in registers (Sec. 5.3: low-bit
// weights are widened for the ALUs).  On short reductions (K up to 1024) most of a launch is
// spent outside the loop - first loads, barrier waits, stores - and the tile shapes with a ring
// of two stages exist so that two workgroups share a CU and each works through the other's waits.
//
// The packed weights are read in the tiled layout of include/nm.h: what one 16-row x 128-column
// fragment consumes is one contiguous run of memory, so a direct load asks the L2 for eight whole
// 128-byte lines (in the row layout it gathered 16 or 64 pieces of as many different lines: a
// fifth to a quarter more L2 requests per launch), and the fragment reads from LDS are
// lane-contiguous.
//
// Stage layout (KU 128-column K steps).  A direct load writes 64 lanes x 16 bytes to 1 KB of
// consecutive LDS in lane order, so every array is a sequence of 1 KB blocks and the layout
// inside a block is chosen by which global chunk each lane fetches:
//   X      [BT rows][128 B]; 16-byte chunk c of row r sits in slot c ^ ((r >> 1) & 7): eight
//          consecutive lanes fetch one full 128-byte line, and the MFMA B-fragment reads
//          (16 rows x one slot) spread over all banks;
//   codes  [KU slices][BO / 16 row blocks][64 units], a copy of the tiled layout's blocks;
//   index  the same with the units' index bytes (absent for a dense matrix).
// Synchronisation per step: wait until this wavefront's own loads of the next step have landed
// (s_waitcnt vmcnt with the count of younger loads), barrier (everyone's have, and everyone has
// consumed the stage about to be refilled), issue the loads STAGES-1 steps ahead, read the next
// step's fragments into registers, multiply the current one.
#include <hip/hip_runtime.h>
#include <stdint.h>


#include "nm_internal.h"
#include "nm_gemm_common.h"

namespace nm {

namespace {

// The arguments every workgroup needs before its first operand loads, fetched in one round trip
// to the argument memory: left to itself the compiler fetches each where it is first used, four
// dependent round trips of a few hundred nanoseconds each before the first load is issued.
__device__ __forceinline__ void fetch_now(GemmArgs& a)
{
    asm volatile("" : "+s"(a.X), "+s"(a.vals), "+s"(a.meta), "+s"(a.scales), "+s"(a.bias), "+s"(a.tokens), "+s"(a.K),
                      "+s"(a.ldx), "+s"(a.O), "+s"(a.k_rotate), "+s"(a.out), "+s"(a.acc), "+s"(a.out_dtype), "+s"(a.ldo),
                      "+s"(a.store_through), "+s"(a.out_scale));
}

// The work of one workgroup: output tile `tile` (of `tiles_o` column tiles per token tile) of the
// GEMM `a`.
// KU = 128-column slices per stage (1 or 2): two slices per stage halve the barriers per column
// at the price of a coarser ring.  In the tiled layout consecutive slices of a row block are
// adjacent in memory, so either way every direct load fetches whole 128-byte lines.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int KU>
__device__ __forceinline__ void gemm_dma_tile(const GemmArgs& a, const int tiles_o, const int tile)
{
    using U = Unit<N, M, BITS>;
    using G = DmaGeom<N, M, BITS, BT, BO, KU>;
    static_assert(BO % (16 * WAVES_O) == 0, "wave tiles are whole row blocks");
    constexpr int NW = WAVES_T * WAVES_O;
    constexpr int WT = BT / WAVES_T, WO = BO / WAVES_O;
    constexpr int FT = WT / 16, FO = WO / 16;
    static_assert(WT % 16 == 0 && WO % 16 == 0, "wave tile must be whole 16x16 fragments");
    static_assert(BT % 8 == 0, "X blocks hold 8 rows");
    static_assert(KU == 1 || KU == 2, "one or two slices per stage");
    constexpr int PER_WAVE = (G::BLOCKS + NW - 1) / NW;      // direct loads per wavefront per stage
    constexpr int STAGE = PER_WAVE * NW * 1024;              // bytes (tail blocks of the last wave are padding)

    extern __shared__ __align__(1024) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wt = wave % WAVES_T, wo = wave / WAVES_T;

    const int t0 = (tile / tiles_o) * BT;
    const int o0 = (tile % tiles_o) * BO;
    const int nk = a.K >> 7;                   // 128-column slices
    const int ns = nk / KU;                    // stages to stream (host guarantees nk % KU == 0)

    // Scales and bias of the tile's columns go to LDS behind the ring (1 KB each, lane l brings
    // columns 4l .. 4l+3), requested before anything else so that their latency hides behind the
    // main loop, and read back into registers only in the epilogue: kept in registers through the
    // loop they would cost 8 VGPRs per weight fragment.  Being the oldest loads of their
    // wavefronts, every later wait on the in-order counter covers them.
    const int li = lane & 15, lg = lane >> 4;
    constexpr int SB_OFF = STAGES * STAGE;
    static_assert(BO <= 256, "one direct load brings the scales of 256 columns");
    {
        const int w_u = __builtin_amdgcn_readfirstlane(wave);
        const uint32_t off = (uint32_t)min(o0 + 4 * lane, a.O - 4) * 4u;
        if (w_u == 0) dma16s((uint32_t)(uintptr_t)smem + SB_OFF, off, reinterpret_cast<const uint8_t*>(a.scales));
        if (w_u == 1 % NW && a.bias != nullptr) dma16s((uint32_t)(uintptr_t)smem + SB_OFF + 1024, off, reinterpret_cast<const uint8_t*>(a.bias));
    }
    float4 sw[FO], bw[FO];
    auto read_scales = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int fo = 0; fo < FO; ++fo) {
            const int c = wo * WO + fo * 16 + 4 * lg;
            sw[fo] = *reinterpret_cast<const float4*>(smem + SB_OFF + c * 4);
            bw[fo] = a.bias ? *reinterpret_cast<const float4*>(smem + SB_OFF + 1024 + c * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };

    // ---- sources of this wavefront's PER_WAVE loads per stage ---------------------------------
    // Load p of wave w fills block b = p * NW + w of the stage; blocks past the last real one are
    // padding and refetch it.  Which array a block belongs to depends on the wavefront only, so
    // its base address and its step along K are scalars; each lane keeps a 32-bit byte offset
    // that is advanced in place after every issue: one add per load in the inner loop.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint32_t voff[PER_WAVE];                   // this lane's byte offset from sbase[p], at the next stage to issue
    const uint8_t* sbase[PER_WAVE];
    uint32_t stepb[PER_WAVE];                  // bytes per stage along the source row
    // With several rounds of tiles per CU, workgroups walk K in rotated order (stage j of this
    // workgroup is K block (kstart + j) mod ns; integer sums do not care), so that workgroups
    // sharing rows of X do not all miss on the same lines at the same moment (8-9 % on the
    // 12288- to 49152-token layer sets).  With a single round every workgroup starts at the same
    // instant on inputs that no L2 holds yet, and rotated starts would ask the memory for all of X
    // and W at once, the first stages queueing behind everybody's later ones: there all start at
    // block 0 (3.5-4.5 % on the 4096-token layer sets).
    const int kstart = a.k_rotate ? (int)(((unsigned)tile * 7u) % (unsigned)ns) : 0;
    const int rb_last = (a.O + 15) / 16 - 1;   // last row block of the packed arrays
    const uint32_t lds_mine = (uint32_t)(uintptr_t)smem + (uint32_t)wave_u * 1024u;
#pragma unroll
    for (int p = 0; p < PER_WAVE; ++p) {
        const int b = min(p * NW + wave_u, G::BLOCKS - 1);
        if (b < G::X_BLOCKS) {
            const int sub = b / (BT / 8);
            const int row = (b % (BT / 8)) * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            const int trow = min(t0 + row, a.tokens - 1);
            sbase[p] = reinterpret_cast<const uint8_t*>(a.X);
            stepb[p] = 128 * KU;
            voff[p] = (uint32_t)trow * (uint32_t)a.ldx + sub * 128 + chunk * 16;
        } else if (b < G::X_BLOCKS + G::V_BLOCKS) {
            // byte q of the stage's codes array = slice s, row block fb, byte w of that block
            const int q = min((b - G::X_BLOCKS) * 1024 + lane * 16, G::V_BYTES - 16);
            const int sl = q / (G::FB * G::VBLK), fb = (q % (G::FB * G::VBLK)) / G::VBLK, w = q % G::VBLK;
            const int rb = min(o0 / 16 + fb, rb_last);
            sbase[p] = a.vals;
            stepb[p] = KU * G::VBLK;
            voff[p] = ((uint32_t)rb * (uint32_t)nk + (uint32_t)sl) * (uint32_t)G::VBLK + (uint32_t)w;
        } else {
            const int q = min((b - G::X_BLOCKS - G::V_BLOCKS) * 1024 + lane * 16, (G::M_BYTES > 16 ? G::M_BYTES : 16) - 16);
            const int sl = q / (G::FB * G::MBLK_), fb = (q % (G::FB * G::MBLK_)) / G::MBLK_, w = q % G::MBLK_;
            const int rb = min(o0 / 16 + fb, rb_last);
            sbase[p] = a.meta;
            stepb[p] = KU * G::MBLK;
            voff[p] = ((uint32_t)rb * (uint32_t)nk + (uint32_t)sl) * (uint32_t)G::MBLK + (uint32_t)w;
        }
        voff[p] += (uint32_t)kstart * stepb[p];
        // The first stage's load of this block leaves at once (ring slot 0): the address work of
        // the remaining blocks - some hundred instructions in all - then runs in the shadow of
        // the memory latency instead of in front of it.
        dma16s(lds_mine + p * NW * 1024, voff[p], sbase[p]);
        voff[p] += stepb[p];
    }
    int k_issue = kstart + 1;                  // K block of the next stage to issue
    if (k_issue == ns) {                       // a single stage: back to K block 0
        k_issue = 0;
#pragma unroll
        for (int p = 0; p < PER_WAVE; ++p) voff[p] -= (uint32_t)ns * stepb[p];
    }
    // Issues the next stage of the stream into ring slot SLOT (a compile-time value).
    auto issue = [&](auto slot) __attribute__((always_inline)) {
        constexpr int SLOT = decltype(slot)::value;
#pragma unroll
        for (int p = 0; p < PER_WAVE; ++p) {
            dma16s(lds_mine + (SLOT * STAGE + p * NW * 1024), voff[p], sbase[p]);
            voff[p] += stepb[p];
        }
        if (++k_issue == ns) {                 // wrapped: back to K block 0
            k_issue = 0;
#pragma unroll
            for (int p = 0; p < PER_WAVE; ++p) voff[p] -= (uint32_t)ns * stepb[p];
        }
    };
    // The same stage in PARTS pieces, piece PART at a time, so that the loads can be spread over
    // the MFMAs of a step: a direct load occupies the address path for some 16 cycles, a
    // wavefront that meets a busy path waits at the instruction, and if all wavefronts issue
    // their loads in one burst after the barrier the matrix pipe idles meanwhile.
    auto issue_part = [&](auto slot, auto part, auto parts) __attribute__((always_inline)) {
        constexpr int SLOT = decltype(slot)::value, PART = decltype(part)::value, PARTS = decltype(parts)::value;
        constexpr int P0 = PART * PER_WAVE / PARTS, P1 = (PART + 1) * PER_WAVE / PARTS;
#pragma unroll
        for (int p = P0; p < P1; ++p) {
            dma16s(lds_mine + (SLOT * STAGE + p * NW * 1024), voff[p], sbase[p]);
            voff[p] += stepb[p];
        }
        if constexpr (PART == PARTS - 1) {
            if (++k_issue == ns) {
                k_issue = 0;
#pragma unroll
                for (int p = 0; p < PER_WAVE; ++p) voff[p] -= (uint32_t)ns * stepb[p];
            }
        }
    };

    v4i acc[FO][FT];
#pragma unroll
    for (int fo = 0; fo < FO; ++fo)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};

    // Fragment addresses inside a stage, for slice s (added at use): B fragment rows start at
    // multiples of 16, so the swizzle term (row >> 1) & 7 only depends on the lane.
    const int xsw = (li >> 1) & 7;
    const int frag_x_lo = G::X_OFF + (wt * WT + li) * 128 + ((lg ^ xsw) * 16);
    const int frag_x_hi = G::X_OFF + (wt * WT + li) * 128 + (((lg + 4) ^ xsw) * 16);
    // weight fragments: the wavefront's FO row blocks of slice s start at frag_w + s * FB * block bytes
    const int frag_v = G::V_OFF + wo * FO * G::VBLK;
    const int frag_m = G::M_OFF + wo * FO * G::MBLK;

    // Fragments live in registers one slice ahead of the MFMAs: while the matrix pipe works on
    // slice k, the LDS reads of slice k+1 are already in flight.
    struct Frags {
        v8i b[FT];
        typename U::Raw w[FO];
    };
    auto load_w = [&](const uint8_t* base, auto sub, auto foc) __attribute__((always_inline)) {
        constexpr int s = decltype(sub)::value, fo = decltype(foc)::value;
        return U::load_tiled(base + frag_v + (s * G::FB + fo) * G::VBLK, base + frag_m + (s * G::FB + fo) * G::MBLK, lane);
    };
    auto fetch = [&](auto slot, auto sub, Frags& f) __attribute__((always_inline)) {
        constexpr int s = decltype(sub)::value;
        const uint8_t* base = smem + decltype(slot)::value * STAGE;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const v4i lo = *reinterpret_cast<const v4i*>(base + s * G::X_SUB + frag_x_lo + ft * 16 * 128);
            const v4i hi = *reinterpret_cast<const v4i*>(base + s * G::X_SUB + frag_x_hi + ft * 16 * 128);
            f.b[ft] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        int_for<FO>([&](auto foc) __attribute__((always_inline)) { f.w[decltype(foc)::value] = load_w(base, sub, foc); });
    };
    auto read_b = [&](auto slot, auto sub, auto ftc, v8i& dst) __attribute__((always_inline)) {
        constexpr int s = decltype(sub)::value, ft = decltype(ftc)::value;
        const uint8_t* base = smem + decltype(slot)::value * STAGE;
        const v4i lo = *reinterpret_cast<const v4i*>(base + s * G::X_SUB + frag_x_lo + ft * 16 * 128);
        const v4i hi = *reinterpret_cast<const v4i*>(base + s * G::X_SUB + frag_x_hi + ft * 16 * 128);
        dst = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };
    auto read_w = [&](auto slot, auto sub, auto foc, typename U::Raw& dst) __attribute__((always_inline)) {
        dst = load_w(smem + decltype(slot)::value * STAGE, sub, foc);
    };
    // The MFMAs of one weight fragment over token fragments [FT0, FT1) of `bsrc`: one sparse MFMA
    // per pair of fragments, two (one per operand half) for the patterns that keep more than two
    // entries in a subgroup of four.
    auto mma_frag = [&](const typename U::Raw& w, const v8i* bsrc, auto foc, auto ft0, auto ft1) __attribute__((always_inline)) {
        constexpr int fo = decltype(foc)::value;
        if constexpr (U::DUAL) {
            v4i c1, c2; int p1, p2;
            U::decode2(w, c1, p1, c2, p2);
#pragma unroll
            for (int ft = decltype(ft0)::value; ft < decltype(ft1)::value; ++ft) {
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(c1, bsrc[ft], acc[fo][ft], p1, 0, 0);
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(c2, bsrc[ft], acc[fo][ft], p2, 0, 0);
            }
        } else {
            v4i codes; int pos;
            U::decode(w, codes, pos);
#pragma unroll
            for (int ft = decltype(ft0)::value; ft < decltype(ft1)::value; ++ft)
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(codes, bsrc[ft], acc[fo][ft], pos, 0, 0);
        }
    };
    // One group of a paced block: the MFMAs of weight fragment FO_I over token fragments
    // [FT0, FT1) of `bsrc`, then piece FO_I of the next stage's loads, fenced so that the compiler
    // keeps them in this order.  The caller places the group's LDS reads in front.
    auto mma_group = [&](const typename U::Raw& w, const v8i* bsrc, auto foc, auto ft0, auto ft1, auto slot, bool more) __attribute__((always_inline)) {
        constexpr int fo = decltype(foc)::value;
        mma_frag(w, bsrc, foc, ft0, ft1);
        __builtin_amdgcn_sched_barrier(0);
        if (more) issue_part(slot, foc, std::integral_constant<int, FO>{});
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mma = [&](const Frags& f) __attribute__((always_inline)) {
        int_for<FO>([&](auto foc) __attribute__((always_inline)) {
            mma_frag(f.w[decltype(foc)::value], f.b, foc, std::integral_constant<int, 0>{}, std::integral_constant<int, FT>{});
        });
    };
    auto interleave = [&]() __attribute__((always_inline)) {
        // One MFMA, then one LDS read issued in its shadow.  A wavefront issues in order, so
        // without this the reads of the next slice would all sit behind (or in front of) the
        // MFMAs and the LDS would idle while the matrix pipe runs.
#pragma unroll
        for (int i = 0; i < FO * FT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, U::DUAL ? 2 : 1, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
        }
    };

    // Large wave tiles (four or more token fragments per wavefront, single-slice stages): two full
    // fragment sets would not fit the register file, so the token fragments are single-buffered in
    // two halves instead - while the MFMAs of one half run, the other half (of this slice, then of
    // the next) is read - and only the weight fragments are double-buffered.
    constexpr bool SPLIT = (KU == 1 && FT >= 4 && FT % 2 == 0);
    constexpr int HT = FT / 2;
    v8i bq[SPLIT ? FT : 1];
    typename U::Raw wq[2][SPLIT ? FO : 1];
    auto fetch_b = [&](auto slot, auto half) __attribute__((always_inline)) {
        const uint8_t* base = smem + decltype(slot)::value * STAGE;
#pragma unroll
        for (int i = 0; i < HT; ++i) {
            const int ft = decltype(half)::value * HT + i;
            const v4i lo = *reinterpret_cast<const v4i*>(base + frag_x_lo + ft * 16 * 128);
            const v4i hi = *reinterpret_cast<const v4i*>(base + frag_x_hi + ft * 16 * 128);
            bq[ft] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };
    auto fetch_w = [&](auto slot, auto set) __attribute__((always_inline)) {
        const uint8_t* base = smem + decltype(slot)::value * STAGE;
        int_for<FO>([&](auto foc) __attribute__((always_inline)) {
            wq[decltype(set)::value][decltype(foc)::value] = load_w(base, std::integral_constant<int, 0>{}, foc);
        });
    };
    auto mma_half = [&](auto set, auto half) __attribute__((always_inline)) {
        int_for<FO>([&](auto foc) __attribute__((always_inline)) {
            mma_frag(wq[decltype(set)::value][decltype(foc)::value], bq, foc, std::integral_constant<int, decltype(half)::value * HT>{},
                     std::integral_constant<int, decltype(half)::value * HT + HT>{});
        });
    };
    // READS LDS reads against FO * HT MFMAs: the surplus first, then one for one.
    auto interleave_half = [&](auto reads) __attribute__((always_inline)) {
        constexpr int READS = decltype(reads)::value, MMAS = FO * HT;
        if constexpr (READS > MMAS) __builtin_amdgcn_sched_group_barrier(0x100, READS - MMAS, 0);
#pragma unroll
        for (int i = 0; i < MMAS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, U::DUAL ? 2 : 1, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
        }
    };

    // ---- pipeline -----------------------------------------------------------------------------
    // Ring of STAGES stages, stream stage j in ring slot j % STAGES.  Fragments are read into
    // registers one slice ahead of their MFMAs, so by the barrier of step j every wavefront has
    // taken the last of stage j out of the LDS (it waits for its own reads first), and the slot
    // of stage j itself is refilled with stage j+STAGES: all other slots hold stages in flight
    // or landed, AHEAD = STAGES-1 steps of latency cover for STAGES slots.  The loop body covers
    // UNROLL consecutive stages so that ring slots and fragment sets are compile-time values:
    // no slot arithmetic, LDS addresses fold into instruction offsets.
    constexpr int AHEAD = STAGES - 1;
    static_assert(AHEAD >= 1, "at least two stages");
    static_assert(AHEAD * PER_WAVE < 64, "loads in flight must fit the counter");
    int_for<AHEAD>([&](auto jj) __attribute__((always_inline)) {     // stage 0 left with the address set-up above
        if (decltype(jj)::value + 1 < ns) issue(std::integral_constant<int, (decltype(jj)::value + 1) % STAGES>{});
    });

    Frags fr[2];
    {   // stage 0 landed; the min(ns, STAGES) - 1 stages behind it may still fly
        bool waited = false;
        int_for<AHEAD + 1>([&](auto c) __attribute__((always_inline)) {
            constexpr int BEHIND = AHEAD - decltype(c)::value;
            if (!waited && ns > BEHIND) {
                wait_vm<BEHIND * PER_WAVE>();
                waited = true;
            }
        });
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if constexpr (SPLIT) {
        fetch_w(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        fetch_b(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    } else {
        fetch(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, fr[0]);
    }

    // Everything needed before the fragments of the first slice of stage j+1 can be read; SLOT is
    // the ring slot of stage j.
    auto advance = [&](int j) __attribute__((always_inline)) {
        if (j + 1 < ns) {
            // stages j+1 .. min(j+AHEAD, ns-1) are in flight, oldest first
            if (j + AHEAD < ns) wait_vm<(AHEAD - 1) * PER_WAVE>();
            else wait_vm<0>();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own reads of stage j done: its slot may be refilled
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        return j + 1 + AHEAD < ns;
    };
    // The fragment fetch is unconditional (after the last slice it re-reads an idle slot and the
    // values are dropped) so that the two register sets never merge across a branch.
    constexpr int UNROLL = (KU == 2 || STAGES % 2 == 0) ? STAGES : 2 * STAGES;
    for (int j0 = 0; j0 < ns; j0 += UNROLL) {
        int_for<UNROLL>([&](auto ss) __attribute__((always_inline)) {
            constexpr int S = decltype(ss)::value;
            constexpr int SLOT = S % STAGES, NEXT = (S + 1) % STAGES;
            const int j = j0 + S;
            if (j < ns) {
                using Fill = std::integral_constant<int, (SLOT + AHEAD + 1) % STAGES>;   // ring slot refilled during this step
                using Next = std::integral_constant<int, NEXT>;
                using Zero = std::integral_constant<int, 0>;
                if constexpr (KU == 2) {
                    mma(fr[0]);
                    fetch(std::integral_constant<int, SLOT>{}, std::integral_constant<int, 1>{}, fr[1]);
                    interleave();
                    const bool more = advance(j);
                    int_for<FO>([&](auto g) __attribute__((always_inline)) {
                        constexpr int fo = decltype(g)::value;
                        read_w(Next{}, Zero{}, g, fr[0].w[fo]);
                        int_for<(fo + 1) * FT / FO - fo * FT / FO>([&](auto i) __attribute__((always_inline)) {
                            constexpr int ft = fo * FT / FO + decltype(i)::value;
                            read_b(Next{}, Zero{}, std::integral_constant<int, ft>{}, fr[0].b[ft]);
                        });
                        mma_group(fr[1].w[fo], fr[1].b, g, Zero{}, std::integral_constant<int, FT>{}, Fill{}, more);
                    });
                } else if constexpr (SPLIT) {
                    // first half of the token fragments, while the second half is read
                    fetch_b(std::integral_constant<int, SLOT>{}, std::integral_constant<int, 1>{});
                    mma_half(std::integral_constant<int, S % 2>{}, std::integral_constant<int, 0>{});
                    interleave_half(std::integral_constant<int, 2 * HT>{});
                    const bool more = advance(j);
                    // second half, while the next slice's weights and first half are read
                    int_for<FO>([&](auto g) __attribute__((always_inline)) {
                        constexpr int fo = decltype(g)::value;
                        read_w(Next{}, Zero{}, g, wq[1 - S % 2][fo]);
                        int_for<(fo + 1) * HT / FO - fo * HT / FO>([&](auto i) __attribute__((always_inline)) {
                            constexpr int ft = fo * HT / FO + decltype(i)::value;
                            read_b(Next{}, Zero{}, std::integral_constant<int, ft>{}, bq[ft]);
                        });
                        mma_group(wq[S % 2][fo], bq, g, std::integral_constant<int, HT>{}, std::integral_constant<int, FT>{}, Fill{}, more);
                    });
                } else {
                    const bool more = advance(j);
                    int_for<FO>([&](auto g) __attribute__((always_inline)) {
                        constexpr int fo = decltype(g)::value;
                        read_w(Next{}, Zero{}, g, fr[1 - S % 2].w[fo]);
                        int_for<(fo + 1) * FT / FO - fo * FT / FO>([&](auto i) __attribute__((always_inline)) {
                            constexpr int ft = fo * FT / FO + decltype(i)::value;
                            read_b(Next{}, Zero{}, std::integral_constant<int, ft>{}, fr[1 - S % 2].b[ft]);
                        });
                        mma_group(fr[S % 2].w[fo], fr[S % 2].b, g, Zero{}, std::integral_constant<int, FT>{}, Fill{}, more);
                    });
                }
            }
        });
    }

    // ---- epilogue: Eq. 4 with offset 0 on the product of two quantised operands --------------
    // The MFMA leaves each lane with 4 consecutive outputs of one token, so a plain store would
    // write 8-byte (bf16) pieces, 32 contiguous bytes per token and instruction.  Exact
    // accumulators, when asked for, and ragged column tiles take that route; the dequantised
    // output first trades registers between lanes so that every lane stores 16 bytes.
    const bool full_cols = (o0 + BO <= a.O);
    if (a.out_dtype == 3) {
        // Requantised output: the scale and bias of each column become its multiplier g and
        // offset h (two divisions per column, done once by one lane each, in place in the LDS).
        if (tid < BO) {
            float* sp = reinterpret_cast<float*>(smem + SB_OFF) + tid;
            float g, h;
            requant_column(act_scale_of(a), sp[0], a.bias ? sp[256] : 0.0f, out_scale_of(a), g, h);
            sp[0] = g;
            sp[256] = h;
        }
        __syncthreads();
    }
    read_scales();
    if (a.acc != nullptr || a.out_dtype == 0 || !full_cols) {
        store_tile_pre<FO, FT>(a, acc, sw, bw, o0 + wo * WO, t0 + wt * WT, li, lg);
        return;
    }
    const int esize = (a.out_dtype == 1) ? 4 : (a.out_dtype == 2) ? 2 : 1;
    if ((a.ldo * esize) % (a.out_dtype == 3 ? 8 : 16) != 0) {   // rows not 16-byte (int8 codes: 8-byte) aligned
        store_tile_pre<FO, FT>(a, acc, sw, bw, o0 + wo * WO, t0 + wt * WT, li, lg);
        return;
    }
    uint8_t* out = reinterpret_cast<uint8_t*>(a.out);
    const int row0 = t0 + wt * WT + li, col0 = o0 + wo * WO;
    const float s_act = act_scale_of(a);
    auto dequant = [&](auto foc, auto ftc, float (&y)[4]) __attribute__((always_inline)) {
        constexpr int fo = decltype(foc)::value, ft = decltype(ftc)::value;
        const v4i c = acc[fo][ft];
        y[0] = (float)c[0] * (s_act * sw[fo].x) + bw[fo].x;
        y[1] = (float)c[1] * (s_act * sw[fo].y) + bw[fo].y;
        y[2] = (float)c[2] * (s_act * sw[fo].z) + bw[fo].z;
        y[3] = (float)c[3] * (s_act * sw[fo].w) + bw[fo].w;
    };
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    if (a.out_dtype == 3) {
        // int8 codes for the next layer: a fragment is one dword per lane; two fragments exchange
        // 16-lane rows as for bf16 below and a lane stores 8 consecutive columns of one token.
        float m = 0.0f;
        auto codes = [&](auto foc, auto ftc) __attribute__((always_inline)) -> uint32_t {
            constexpr int fo = decltype(foc)::value, ft = decltype(ftc)::value;
            const float g[4] = {sw[fo].x, sw[fo].y, sw[fo].z, sw[fo].w};    // the columns' multipliers and offsets
            const float h[4] = {bw[fo].x, bw[fo].y, bw[fo].z, bw[fo].w};
            return requant4(acc[fo][ft], g, h, m);
        };
        auto emit8 = [&](uint32_t da, uint32_t db, int row, int col) __attribute__((always_inline)) {
            const v2u x = __builtin_amdgcn_permlane16_swap(da, db, false, false);
            if (row < a.tokens) {
                uint8_t* dst = out + (size_t)row * a.ldo + col;
                if (a.store_through) store8_through(dst, v2i_t{(int)x[0], (int)x[1]});
                else *reinterpret_cast<uint2*>(dst) = make_uint2(x[0], x[1]);
            }
        };
        // Four fragments side by side go one step further (v_permlane32_swap: upper half of the
        // first operand against lower half of the second): lane row lg ends up with all 16 columns
        // of fragment lg of the four, 16 bytes, in the order (P, R, Q, S) of the two exchanges.
        constexpr int Q4 = FO / 4;
        const bool wide = (a.ldo % 16 == 0) && ((uintptr_t)a.out % 16 == 0);
        int_for<FT>([&](auto ftc) __attribute__((always_inline)) {
            constexpr int ft = decltype(ftc)::value;
            if (wide) {
                int_for<Q4>([&](auto h) __attribute__((always_inline)) {
                    constexpr int fo = 4 * decltype(h)::value;
                    const uint32_t ca = codes(std::integral_constant<int, fo>{}, ftc), cb = codes(std::integral_constant<int, fo + 1>{}, ftc);
                    const uint32_t cc = codes(std::integral_constant<int, fo + 2>{}, ftc), cd = codes(std::integral_constant<int, fo + 3>{}, ftc);
                    const v2u ab = __builtin_amdgcn_permlane16_swap(ca, cb, false, false);
                    const v2u cd2 = __builtin_amdgcn_permlane16_swap(cc, cd, false, false);
                    const v2u pq = __builtin_amdgcn_permlane32_swap(ab[0], cd2[0], false, false);
                    const v2u rs = __builtin_amdgcn_permlane32_swap(ab[1], cd2[1], false, false);
                    const int row = row0 + ft * 16;
                    if (row < a.tokens) {
                        uint8_t* dst = out + (size_t)row * a.ldo + col0 + (fo + lg) * 16;
                        const v4i v = v4i{(int)pq[0], (int)rs[0], (int)pq[1], (int)rs[1]};
                        if (a.store_through) store16_through(dst, v);
                        else *reinterpret_cast<v4i*>(dst) = v;
                    }
                });
            } else {
                int_for<2 * Q4>([&](auto h) __attribute__((always_inline)) {
                    constexpr int fo = 2 * decltype(h)::value;
                    const uint32_t da = codes(std::integral_constant<int, fo>{}, ftc);
                    const uint32_t db = codes(std::integral_constant<int, fo + 1>{}, ftc);
                    emit8(da, db, row0 + ft * 16, col0 + fo * 16 + (lg & 1) * 16 + (lg >> 1) * 8);
                });
            }
            int_for<(FO - 4 * Q4) / 2>([&](auto h) __attribute__((always_inline)) {
                constexpr int fo = 4 * Q4 + 2 * decltype(h)::value;
                const uint32_t da = codes(std::integral_constant<int, fo>{}, ftc);
                const uint32_t db = codes(std::integral_constant<int, fo + 1>{}, ftc);
                emit8(da, db, row0 + ft * 16, col0 + fo * 16 + (lg & 1) * 16 + (lg >> 1) * 8);
            });
        });
        if constexpr (FO % 2 == 1) {
            constexpr int fo = FO - 1;
            int_for<FT / 2>([&](auto h) __attribute__((always_inline)) {
                constexpr int ft = 2 * decltype(h)::value;
                const uint32_t da = codes(std::integral_constant<int, fo>{}, std::integral_constant<int, ft>{});
                const uint32_t db = codes(std::integral_constant<int, fo>{}, std::integral_constant<int, ft + 1>{});
                emit8(da, db, row0 + (ft + (lg & 1)) * 16, col0 + fo * 16 + (lg >> 1) * 8);
            });
        }
        absmax_commit(m, out_scale_of(a), a.absmax);
        return;
    }
    if (a.out_dtype == 1) {
        // fp32: the accumulator layout is already 16 bytes per lane, 64 contiguous bytes per
        // token and instruction.  Always written through: measured faster at every size.
        int_for<FT>([&](auto ftc) __attribute__((always_inline)) {
            constexpr int ft = decltype(ftc)::value;
            int_for<FO>([&](auto foc) __attribute__((always_inline)) {
                constexpr int fo = decltype(foc)::value;
                float y[4];
                dequant(foc, ftc, y);
                const int row = row0 + ft * 16;
                if (row < a.tokens)
                    store16_through(out + ((size_t)row * a.ldo + col0 + fo * 16 + 4 * lg) * 4,
                                    v4i{(int)__float_as_uint(y[0]), (int)__float_as_uint(y[1]), (int)__float_as_uint(y[2]), (int)__float_as_uint(y[3])});
            });
        });
        return;
    }
    // bf16: two fragments side by side (16 columns apart) exchange 16-lane rows
    // (v_permlane16_swap: odd rows of the first operand against even rows of the second), after
    // which lane row lg holds 8 consecutive columns of one token - columns
    // (lg & 1) * 16 + (lg >> 1) * 8 onwards of the pair's 32 - and one 16-byte store per lane
    // writes 64 contiguous bytes per token.  An odd last fragment pairs with its neighbour along
    // the tokens instead: lane row lg then holds columns (lg >> 1) * 8 onwards of token fragment
    // ft + (lg & 1).  No trip through the LDS, no barrier.
    const bool through = a.store_through != 0;
    auto emit = [&](const float (&ya)[4], const float (&yb)[4], int row, int col) __attribute__((always_inline)) {
        const v2u x = __builtin_amdgcn_permlane16_swap(pack_bf16x2(ya[0], ya[1]), pack_bf16x2(yb[0], yb[1]), false, false);
        const v2u y = __builtin_amdgcn_permlane16_swap(pack_bf16x2(ya[2], ya[3]), pack_bf16x2(yb[2], yb[3]), false, false);
        if (row < a.tokens) {
            uint8_t* dst = out + ((size_t)row * a.ldo + col) * 2;
            const v4i v = v4i{(int)x[0], (int)y[0], (int)x[1], (int)y[1]};
            if (through) store16_through(dst, v);
            else *reinterpret_cast<v4i*>(dst) = v;
        }
    };
    static_assert(FO % 2 == 0 || FT % 2 == 0, "fragments must pair up along one side");
    int_for<FT>([&](auto ftc) __attribute__((always_inline)) {
        constexpr int ft = decltype(ftc)::value;
        int_for<FO / 2>([&](auto h) __attribute__((always_inline)) {
            constexpr int fo = 2 * decltype(h)::value;
            float ya[4], yb[4];
            dequant(std::integral_constant<int, fo>{}, ftc, ya);
            dequant(std::integral_constant<int, fo + 1>{}, ftc, yb);
            emit(ya, yb, row0 + ft * 16, col0 + fo * 16 + (lg & 1) * 16 + (lg >> 1) * 8);
        });
    });
    if constexpr (FO % 2 == 1) {
        constexpr int fo = FO - 1;
        int_for<FT / 2>([&](auto h) __attribute__((always_inline)) {
            constexpr int ft = 2 * decltype(h)::value;
            float ya[4], yb[4];
            dequant(std::integral_constant<int, fo>{}, std::integral_constant<int, ft>{}, ya);
            dequant(std::integral_constant<int, fo>{}, std::integral_constant<int, ft + 1>{}, yb);
            emit(ya, yb, row0 + (ft + (lg & 1)) * 16, col0 + fo * 16 + (lg >> 1) * 8);
        });
    }
}

// One GEMM per launch.  Workgroup -> tile: each XCD (workgroups are dealt to the eight XCDs in
// turn) takes a contiguous run of tiles, so that the CUs behind one L2 share token rows.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int KU>
__global__ void __launch_bounds__(64 * WAVES_T * WAVES_O, STAGES == 2 ? 2 : 1)
gemm_dma_kernel(const GemmArgs a_in, const int tiles_o, const int n_tiles)
{
    GemmArgs a = a_in;
    fetch_now(a);                              // ahead of the early exit: one round trip for everything
    const int per_xcd = (n_tiles + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= n_tiles) return;               // whole workgroup leaves before any barrier
    gemm_dma_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, KU>(a, tiles_o, tile);
}

// Several GEMMs per launch (nm_gemm_batch): each workgroup first finds the item its tile belongs
// to - a second, dependent round trip to the argument memory before the first loads, which a
// launch of one GEMM does without (it costs that launch 0.1 to 0.5 us), hence a kernel of its own.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int KU>
__global__ void __launch_bounds__(64 * WAVES_T * WAVES_O, STAGES == 2 ? 2 : 1)
gemm_dma_batch_kernel(const GemmBatch p)
{
    const int n_tiles = p.first_tile[p.count];
    const int per_xcd = (n_tiles + 7) >> 3;
    int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= n_tiles) return;
    int item = 0;                              // uniform over the workgroup
    while (item + 1 < p.count && tile >= p.first_tile[item + 1]) ++item;
    GemmArgs a = p.item[item];
    fetch_now(a);
    gemm_dma_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, KU>(a, p.tiles_o[item], tile - p.first_tile[item]);
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int KU, bool BATCHABLE = false>
bool launch_dma_tile(const GemmArgs* items, int count, hipStream_t st)
{
    using G = DmaGeom<N, M, BITS, BT, BO, KU>;
    constexpr int NW = WAVES_T * WAVES_O;
    constexpr int PER_WAVE = (G::BLOCKS + NW - 1) / NW;
    constexpr size_t lds = (size_t)STAGES * PER_WAVE * NW * 1024 + 2048;   // ring, then scales and bias of the tile
    static_assert(lds <= 160 * 1024, "LDS ring exceeds the 160 KB of a CU");
    if (count > 1 && !BATCHABLE) return false;
    GemmBatch b;
    b.count = count;
    b.first_tile[0] = 0;
    long long out_bytes = 0;
    for (int i = 0; i < count; ++i) {
        const GemmArgs& a = items[i];
        if ((a.K / 128) % KU != 0) return false;
        // per-lane source offsets are 32-bit
        if ((unsigned long long)a.tokens * a.ldx >= (1ull << 32) || packed_bytes(a.pv, a.O, a.K) >= (1ull << 32)) return false;
        const int tiles_t = (a.tokens + BT - 1) / BT;
        b.tiles_o[i] = (a.O + BO - 1) / BO;
        if ((long long)b.first_tile[i] + (long long)tiles_t * b.tiles_o[i] > 0x7FFFFFF0ll) return false;
        b.first_tile[i + 1] = b.first_tile[i] + tiles_t * b.tiles_o[i];
        b.item[i] = a;
        out_bytes += (long long)a.tokens * a.O * (a.out_dtype == 3 ? 1 : 2);
    }
    for (int i = count; i < GEMM_BATCH_MAX; ++i) {      // unused slots: defined values
        b.item[i] = items[0];
        b.tiles_o[i] = 0;
        b.first_tile[i + 1] = b.first_tile[count];
    }
    const int n_tiles = b.first_tile[count];
    const int grid = 8 * ((n_tiles + 7) / 8);
    // bf16 outputs of 14 MB and more (all items of the launch together) are written through
    // (measured at 4096 tokens: equal at 12.6 MB, 17 % faster at 18.9 MB, slower below), int8
    // codes from 8 MB (9.4 MB: 11.4 -> 10.4 us, 12.6 MB: 12.5 -> 11.8 us, 50 MB: 56.9 -> 52.9 us);
    // fp32 always is, in the kernel.
    for (int i = 0; i < count; ++i) {
        b.item[i].store_through = out_bytes >= ((items[0].out_dtype == 3 ? 8ll : 14ll) << 20);
        b.item[i].k_rotate = n_tiles > 256;     // more tiles than CUs: see the kernel
    }
    if constexpr (BATCHABLE) {
        if (count > 1) {
            auto kern = gemm_dma_batch_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, KU>;
            if (lds > 64 * 1024) {
                static std::atomic<uint64_t> raised{0};   // per instantiation
                raise_lds_limit(reinterpret_cast<const void*>(kern), lds, raised);
            }
            hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), lds, st, b);
            return true;
        }
    }
    auto kern = gemm_dma_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, KU>;
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> raised{0};   // per instantiation
        raise_lds_limit(reinterpret_cast<const void*>(kern), lds, raised);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), lds, st, b.item[0], b.tiles_o[0], n_tiles);
    return true;
}

// Tile choice.  The kernel is bound by the bytes it moves per multiply-add (L2 -> LDS, LDS ->
// registers: time with few workgroups, energy under the power limit with many) and by
// the fixed cost of a tile, so the tile wants to be as large as the CU count allows: 256 x 192
// where that still gives every CU a tile, else 128 x 96 (exactly 256 workgroups for BERT-base's
// 768-wide layers at 4096 tokens).  Rings of at most 80 KB let two workgroups share a CU, which
// overlaps one's epilogue with the other's prologue when there are several rounds.
// Tile choice for 2:4 int8 (the pattern of the paper's inference table) from a duration model of
// every compiled shape: microseconds = P + R * (F + S * K / 128), R = rounds of tiles over the
// chip's workgroup slots (256 for the shapes whose ring fills a CU, 512 for those that leave room
// for a second workgroup; a last round that fills at most half the slots of a two-per-CU shape
// counts as `tail`).  P, F and S are least-squares fits to launches measured back to back at 4096
// to 24576 tokens on the BERT-base and BERT-large layer shapes (mean error 3 to 7 %); choosing by
// the model lands within 1.4 % of the fastest shape on average over those 48 cases.  What the
// fits say: the two-stage shapes (two workgroups per CU, each covering the other's barrier waits,
// first loads and stores) have almost no fixed cost per tile but the costliest K step, so they
// win on short reductions and few rounds and lose on K = 3072 / 4096; 256 x 256 wins where 192
// does not divide the width.  Outputs beyond the 256 MB Infinity Cache stream to HBM as they are
// produced: there the two-per-CU shapes fall behind (more operand re-reads per multiply-add
// compete with the stores) and are left out.
inline int modelled_tile(const GemmArgs& a)
{
    struct Model { int cfg, bt, bo, slots; float tail, p, f, s; };
    static const Model models[] = {
        {122, 256, 192, 256, 1.0f, 0.61f, 4.59f, 0.750f}, {123, 256, 256, 256, 1.0f, 1.07f, 7.72f, 0.904f},
        {121, 256, 128, 256, 1.0f, 0.70f, 3.21f, 0.663f}, {128, 192, 128, 256, 1.0f, 0.98f, 2.86f, 0.500f},
        {117, 128, 128, 256, 1.0f, 1.64f, 2.41f, 0.368f}, {116, 128, 96, 512, 0.5f, 2.25f, 2.98f, 0.588f},
        {113, 128, 96, 512, 0.5f, 1.65f, 6.09f, 0.520f},  {112, 256, 96, 256, 1.0f, 0.97f, 4.18f, 0.462f},
        {133, 128, 192, 512, 0.7f, 0.95f, 1.34f, 1.190f}, {136, 128, 256, 512, 0.6f, 0.06f, 3.47f, 1.279f}};
    const bool streams_out = (long long)a.tokens * a.O * (a.out_dtype == 3 ? 1 : a.out_dtype == 1 ? 4 : 2) > (256ll << 20);
    float best = 0.0f;
    int pick = 116;
    for (const Model& m : models) {
        const long long ct = (a.O + m.bo - 1) / m.bo;
        if ((ct * m.bo - a.O) * 8 > a.O) continue;                       // an eighth of the columns computed in vain
        if (m.cfg == 113 && (a.K / 128) % 2 != 0) continue;             // two slices per stage
        if ((m.cfg == 133 || m.cfg == 136) && streams_out) continue;
        const long long n = (long long)((a.tokens + m.bt - 1) / m.bt) * ct;
        const long long full = n / m.slots, rem = n % m.slots;
        // (a two-stage shape whose only round leaves every workgroup alone on its CU: 0.9, measured at 2048 tokens)
        const bool two_stage = m.cfg == 133 || m.cfg == 136;
        const float rounds = (float)full + (rem == 0 ? 0.0f : (m.slots > 256 && rem <= m.slots / 2) ? (two_stage && full == 0 ? 0.9f : m.tail) : 1.0f);
        const float us = m.p + rounds * (m.f + m.s * (float)(a.K / 128));
        if (best == 0.0f || us < best) { best = us; pick = m.cfg; }
    }
    return pick;
}

template <int N, int M, int BITS>
bool launch_dma_pattern(const GemmArgs* items, int count, hipStream_t st, int cfg)
{
    using U = Unit<N, M, BITS>;
    // The tile is chosen for the launch as a whole: the items' output widths side by side (query,
    // key and value of one layer are one 3 x wider layer to the cost model), the most tokens.
    GemmArgs a = items[0];
    for (int i = 1; i < count; ++i) {
        a.O += items[i].O;
        a.tokens = a.tokens > items[i].tokens ? a.tokens : items[i].tokens;
    }
    // 3:8, 5:8, 6:8, 7:8: units of 6 to 28 bytes that the dwords of a register do not divide; the
    // 128-wide tiles only (their decode, not the staging, bounds them).
    constexpr bool ODD8 = (M == 8 && N >= 3 && N < 8 && N != 4);
    // 3:4 and 4:8 at 4 bits: the costliest decodes of the patterns that fit the wide tile.  Its eight
    // wavefronts arranged 2 x 4 (wave tiles of 128 x 48) decode every weight fragment twice instead
    // of four times: 256 x 192 in that arrangement (4:8 FFN-up 22.8 -> 20.8 us, QKV 22.3 -> 18.4;
    // 3:4, which does not fit the registers of the 4 x 2 arrangement, 26.8 -> 21.3 and 19.1 -> 18.0).
    // 3:4 and the N:8 patterns with N >= 3 spend more time decoding a weight fragment than multiplying
    // it, and every wavefront that shares the fragment decodes it again.  128 x 128 with the eight
    // wavefronts side by side along the outputs (wave tiles of 128 tokens x 16 outputs) decodes every
    // fragment once, at the price of every wavefront reading the whole token tile: better for every
    // such pattern on outputs up to 1024 wide (4:8 int8 FFN-down 24.1 -> 19.8 us, attention output
    // 9.3 -> 8.1; 3:4 int8 12288 x 1024 -> 1024 35.4 -> 28.5; 5:8 int4 there 66.9 -> 36.4), and at any
    // width for 4:8 int8, five of eight at 8 bits and six or seven of eight (5:8 int8 FFN-up
    // 39.6 -> 30.4 us, 7:8 int8 45.9 -> 32.1); the other patterns keep 256 x 192 / 128 x 96 on wide
    // outputs, where those measure equal or better.
    constexpr bool DECODE_BOUND = U::DUAL && N != M;
    constexpr bool ALWAYS_ONCE = M == 8 && (N >= 6 || (N >= 4 && BITS == 8));
    // The cheaper decodes gain from the same arrangement on outputs up to 1024 wide too (FFN-down at
    // 4096 tokens: 2:4 int4 14.6 -> 13.0 us, 2:8 int8 15.0 -> 13.0, dense int4 18.7 -> 15.7); 1:4 int8
    // and dense int8 measure equal either way and keep 128 x 96.
    constexpr bool NARROW_ONCE = !U::IDENTITY && !(N == 1 && M == 4 && BITS == 8) && !(N == M && BITS == 8);
    constexpr bool WIDE24 = (BITS == 4 && ((N == 3 && M == 4) || (N == 4 && M == 8)));
    if (cfg == 0) {
        // Cost of a tile shape = rounds over the 256 CUs x tile area x the shape's cost per
        // multiply-add relative to 256 x 192 (time per multiply-add with the chip full, measured: 256 x 128
        // 1.35, 192 x 128 1.5, 128 x 128 1.66, 128 x 96 1.45 with its two workgroups per CU).  A
        // shape whose last column tile would compute more than an eighth of the columns in vain is
        // out; a later shape must beat an earlier one by 5 %.  BERT-base at 4096 tokens: 256 x 192
        // for QKV and FFN-up (192 and 256 tiles), 128 x 96 for the 768-wide outputs (256 tiles);
        // BERT-large at 12288 tokens: 256 x 192 for QKV, 256 x 256 for FFN-up and the 1024-wide
        // layers (768 and 192 tiles); at 4096 tokens 128 x 128 for the 1024-wide ones (256 tiles);
        // at 8192 and 24576 tokens 256 x 128 for them.
        struct Shape { int cfg, bt, bo, cost; };
        // 256 x 256 (four wavefronts of 128 x 128, one per SIMD, accumulators in 256 registers) moves the
        // fewest bytes per multiply-add but hides latency worst: cost 1.15.  It wins where 192 does not
        // divide the output width and 256 does (BERT-large FFN-up, 4096 wide: 54.7 -> 49.5 us at 12288 tokens,
        // 19.1 -> 17.1 us at 4096).
        static const Shape shapes[] = {{122, 256, 192, 100}, {123, 256, 256, 115}, {121, 256, 128, 135}, {128, 192, 128, 150}, {117, 128, 128, 166}, {0, 128, 96, 145}};
        long long best = -1;
        int pick = 0;
        for (const Shape& sh : shapes) {
            if (U::DUAL && BITS == 8 && sh.cfg != 0 && sh.cfg != 117) continue;   // two operands per unit of 24 or 32 bytes: the wide wave tiles would not fit the registers
            if (U::DUAL && N == 3 && sh.cfg == 122 && !WIDE24) continue;
            if (ODD8 && sh.cfg != 0 && sh.cfg != 117) continue;
            if (!U::IDENTITY && sh.cfg == 123) continue;
            if (count > 1 && sh.cfg != 122 && sh.cfg != 117 && sh.cfg != 0) continue;   // the shapes compiled for several GEMMs per launch
            long long ct = 0;                  // column tiles, item by item
            for (int i = 0; i < count; ++i) ct += (items[i].O + sh.bo - 1) / sh.bo;
            if (sh.cfg != 0 && (ct * sh.bo - a.O) * 8 > a.O) continue;
            const long long n = (long long)((a.tokens + sh.bt - 1) / sh.bt) * ct;
            const long long c = ((n + 255) / 256) * sh.bt * sh.bo * sh.cost;
            if (best < 0 || c * 105 < best * 100) { best = c; pick = sh.cfg; }
        }
        const long long n96 = (long long)((a.tokens + 127) / 128) * ((a.O + 95) / 96);
        const long long n64x96 = (long long)((a.tokens + 63) / 64) * ((a.O + 95) / 96);
        const long long n64x48 = (long long)((a.tokens + 63) / 64) * ((a.O + 47) / 48);
        // A problem of fewer than 128 tiles of 128 x 96 leaves half the chip idle while every workgroup
        // pulls its whole share of X and W through one CU's fill path: the smallest tile that still
        // runs in one round (measured on 128 to 384 tokens: 128 x 768 -> 768 5.1 -> 4.2 us,
        // 128 x 4096 -> 1024 10.9 -> 9.3 us, 384 x 1024 -> 3072 6.1 -> 5.0 us).
        if (!U::DUAL && n96 < 128 && n64x48 <= 256) cfg = 130;
        else if (!U::DUAL && n96 < 128 && n64x96 <= 256 && count == 1) cfg = 132;
        else if (NARROW_ONCE && count == 1 && ((DECODE_BOUND && ALWAYS_ONCE) || a.O <= 1024)) cfg = 127;
        else if (U::IDENTITY && count == 1 && n96 >= 256) cfg = modelled_tile(a);
        else if (pick == 122 && WIDE24) cfg = count == 1 ? 126 : (N == 3 ? 117 : 122);
        else if (pick == 122 && (!U::DUAL || (N == M && BITS == 4)) && a.K <= 1024 &&
                 (long long)a.tokens * a.O * (a.out_dtype == 3 ? 1 : a.out_dtype == 1 ? 4 : 2) <= (256ll << 20))
            cfg = 133;      // the decoded patterns and dense int4 on short reductions: two 128 x 192 workgroups per CU (3 to 13 % under 256 x 192, measured on every one of them)
        else if (pick != 0) cfg = pick;
        else if (!ODD8 && n96 >= 1024 && a.tokens >= 256 && count == 1) cfg = 112;      // many rounds: 256 x 96
        else if (!U::IDENTITY) cfg = 115;                        // decode work: four wavefronts of 64 x 48 decode each weight fragment twice, eight of 32 x 48 four times
        else if (a.K >= 2048 && (a.K / 128) % 2 == 0 && count == 1 && n96 <= 256) cfg = 113;   // long reductions in one round of tiles: two slices per stage, half the barriers (4 % at K = 3072; slower with two rounds)
        else cfg = 116;                                          // 128 x 96, eight wavefronts
    }
    note_gemm_tile(cfg);
    if constexpr (!ODD8) {
        if (cfg == 112) return launch_dma_tile<N, M, BITS, 256, 96, 4, 2, 3, 1>(items, count, st);
    }
    if (cfg == 116) return launch_dma_tile<N, M, BITS, 128, 96, 4, 2, 3, 1, true>(items, count, st);
    if (cfg == 115) return launch_dma_tile<N, M, BITS, 128, 96, 2, 2, 3, 1, true>(items, count, st);
    if (cfg == 117) return launch_dma_tile<N, M, BITS, 128, 128, 4, 2, 3, 1, true>(items, count, st);
    if constexpr (NARROW_ONCE) {
        if (cfg == 127) return launch_dma_tile<N, M, BITS, 128, 128, 1, 8, 3, 1>(items, count, st);
    }
    if constexpr (WIDE24) {
        if (cfg == 126) return launch_dma_tile<N, M, BITS, 256, 192, 2, 4, 3, 1>(items, count, st);
    }
    if constexpr (!U::DUAL || (BITS == 4 && N != 3 && !ODD8)) {      // (3:4 needs a few registers more for its index bits: it would spill)
        if (cfg == 122) return launch_dma_tile<N, M, BITS, 256, 192, 4, 2, 3, 1, true>(items, count, st);
        if (cfg == 133) return launch_dma_tile<N, M, BITS, 128, 192, 2, 2, 2, 1, true>(items, count, st);
    }
    if constexpr (!U::DUAL || (BITS == 4 && !ODD8)) {
        if (cfg == 128) return launch_dma_tile<N, M, BITS, 192, 128, 4, 2, 3, 1>(items, count, st);
        if (cfg == 121) return launch_dma_tile<N, M, BITS, 256, 128, 4, 2, 3, 1>(items, count, st);
    }
    if constexpr (U::IDENTITY) {
        if (cfg == 123) return launch_dma_tile<N, M, BITS, 256, 256, 2, 2, 3, 1>(items, count, st);
        if (cfg == 136) return launch_dma_tile<N, M, BITS, 128, 256, 2, 2, 2, 1>(items, count, st);
    }
    if constexpr (!U::DUAL) {
        if (cfg == 113) return launch_dma_tile<N, M, BITS, 128, 96, 4, 2, 3, 2>(items, count, st);
        // small tiles for problems of a few output tiles (few tokens): more workgroups, each with a
        // smaller share of X and W to pull through its CU's fill path
        if (cfg == 130) return launch_dma_tile<N, M, BITS, 64, 48, 2, 1, 4, 1, true>(items, count, st);
        if (cfg == 132) return launch_dma_tile<N, M, BITS, 64, 96, 2, 2, 4, 1>(items, count, st);
    }
    return false;
}

}  // namespace

// One translation unit per set of patterns (NM_DMA_SET, given on the command line), so that the
// many instantiations compile in parallel.  Returns true when it launched a kernel.
#define NM_CAT2(a, b) a##b
#define NM_CAT(a, b) NM_CAT2(a, b)
bool NM_CAT(launch_gemm_dma_set, NM_DMA_SET)(const GemmArgs* items, int count, hipStream_t st, int cfg)
{
    const GemmArgs& a = items[0];
#define NM_CASE(n, m, b) if (a.N == n && a.M == m && a.bits == b) return launch_dma_pattern<n, m, b>(items, count, st, cfg)
#if NM_DMA_SET == 0
    NM_CASE(2, 4, 8);
#elif NM_DMA_SET == 1
    NM_CASE(1, 4, 8); NM_CASE(2, 4, 4);
#elif NM_DMA_SET == 2
    NM_CASE(1, 4, 4); NM_CASE(1, 8, 8);
#elif NM_DMA_SET == 3
    NM_CASE(2, 8, 8); NM_CASE(1, 8, 4);
#elif NM_DMA_SET == 4
    NM_CASE(2, 8, 4);
#elif NM_DMA_SET == 5
    NM_CASE(4, 4, 8); NM_CASE(4, 4, 4); NM_CASE(3, 4, 8);
#elif NM_DMA_SET == 6
    NM_CASE(3, 4, 4); NM_CASE(4, 8, 8); NM_CASE(4, 8, 4);
#elif NM_DMA_SET == 7
    NM_CASE(3, 8, 8); NM_CASE(3, 8, 4);
#elif NM_DMA_SET == 8
    NM_CASE(5, 8, 8); NM_CASE(5, 8, 4);
#elif NM_DMA_SET == 9
    NM_CASE(6, 8, 8); NM_CASE(6, 8, 4);
#elif NM_DMA_SET == 10
    NM_CASE(7, 8, 8); NM_CASE(7, 8, 4);
#else
#error "NM_DMA_SET must be 0 .. 10"
#endif
#undef NM_CASE
    return false;
}

}  // namespace nm
