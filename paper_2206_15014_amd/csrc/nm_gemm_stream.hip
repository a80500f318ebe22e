// nm_gemm, persistent LDS-direct variant for gfx950.
//
// One workgroup per CU walks a list of output tiles.  The operand ring (global_load_lds_dwordx4
// into STAGES stages, as in the one-tile-per-workgroup kernel) never drains between tiles: while
// the last K steps of a tile are multiplied, the first stages of the next tile are already in
// flight, so the memory latency at the head of a tile and the write latency at its tail are paid
// once per launch instead of once per tile.
//
// Memory instructions are split by wavefront.  The lower half of the wavefronts issues every
// load (all of them direct-to-LDS, including the row scales and biases of each tile), the upper
// half issues every store: the dequantised tile (Eq. 4, offset 0) is turned round through an LDS
// staging area and written as whole rows by the upper half.  The in-order memory counter of a
// wavefront counts loads and stores alike, so a wavefront that did both would have to wait for
// its slow stores whenever it waits for the next stage of operands.
//
// Handles the common case only (dequantised output without the exact accumulators, whole column
// tiles, 16-byte aligned output rows); everything else goes to the other kernels.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "nm_gemm_common.h"

namespace nm {

namespace {

// EP = number of passes in which a tile goes through the staging area (BT / EP rows at a time);
// ES = bytes per output element (4: fp32, 2: bf16).
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int EP, int ES>
struct StreamGeom {
    using G = DmaGeom<N, M, BITS, BT, BO, 1>;
    static constexpr int NW = WAVES_T * WAVES_O;
    static constexpr int LW = NW / 2;                                   // loading wavefronts 0 .. LW-1
    static constexpr int SW = NW - LW;                                  // storing wavefronts LW .. NW-1
    static constexpr int PER_LW = (G::BLOCKS + LW - 1) / LW;            // direct loads per loading wavefront per stage
    static constexpr int STAGE = PER_LW * LW * 1024;
    static constexpr int RING = STAGES * STAGE;
    static constexpr int SB_BLOCKS = (2 * BO * 4 + 1023) / 1024;        // scales then biases of a tile
    static constexpr int SB_BYTES = SB_BLOCKS * 1024;
    static constexpr int SB_OFF = RING;                                 // STAGES buffers, one per tile in flight
    static constexpr int ST_OFF = SB_OFF + STAGES * SB_BYTES;
    static constexpr int SROWS = BT / EP;
    static constexpr int SROW_B = BO * ES + 16;                         // staged row stride (the pad spreads banks)
    static constexpr int LDS = ST_OFF + SROWS * SROW_B;
    static_assert(NW % 2 == 0, "half of the wavefronts load, half store");
    static_assert(!G::PAIR_V && !G::PAIR_M, "whole 16-byte rows per stage only");
    static_assert(LDS <= 160 * 1024, "exceeds the 160 KB of LDS of a CU");
};

// Workgroup barriers as one opaque instruction group each.  (__syncthreads() would also wait for
// the vector-memory counter, i.e. for every load or store the wavefront has in flight, which is
// exactly what the ring must not do.)  The first form orders nothing but execution; the second
// first drains this wavefront's LDS operations, for barriers that publish LDS writes.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void wg_barrier_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int EP, int ES>
__global__ void __launch_bounds__(64 * WAVES_T * WAVES_O)
gemm_stream_kernel(const GemmArgs a, const int tiles_o, const int n_tiles)
{
    using U = Unit<N, M, BITS>;
    using S = StreamGeom<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, EP, ES>;
    using G = typename S::G;
    constexpr int NW = S::NW, LW = S::LW, SW = S::SW, PER_LW = S::PER_LW, STAGE = S::STAGE;
    constexpr int WT = BT / WAVES_T, WO = BO / WAVES_O;
    constexpr int FT = WT / 16, FO = WO / 16;
    static_assert(WT % 16 == 0 && WO % 16 == 0, "wave tile must be whole 16x16 fragments");
    static_assert(FT % EP == 0, "every pass takes the same number of fragment rows of each wavefront");
    static_assert(BT % 8 == 0 && BO % 4 == 0, "X blocks hold 8 rows; scales travel in 16-byte pieces");
    constexpr int AHEAD = STAGES - 2;
    static_assert(AHEAD >= 1, "at least three stages");
    static_assert(AHEAD * PER_LW + S::SB_BLOCKS < 64, "loads in flight must fit the counter");

    extern __shared__ __align__(1024) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool loader = wave_u < LW;
    const int wt = wave % WAVES_T, wo = wave / WAVES_T;
    const int li = lane & 15, lg = lane >> 4;

    // ---- tiles of this workgroup ---------------------------------------------------------------
    // Consecutive workgroup ids land on different XCDs (each with its own L2), so tiles are dealt
    // out per XCD: XCD x owns a contiguous range of tiles, and its workgroups walk that range side
    // by side (tile = first + wi, first + wi + gx, ...), which keeps the X rows and the packed
    // weights they share in that XCD's L2.
    const int gx = (int)(gridDim.x >> 3);
    const int xcd = (int)(blockIdx.x & 7), wi = (int)(blockIdx.x >> 3);
    const int per_xcd = (n_tiles + 7) >> 3;
    const int first = xcd * per_xcd + wi;
    const int last = min((xcd + 1) * per_xcd, n_tiles);
    if (first >= last) return;                                // whole workgroup leaves before any barrier
    const int cnt = (last - first + gx - 1) / gx;
    const int ns = a.K >> 7;                                  // stages (128-column slices) per tile
    const int total = cnt * ns;                               // stages this workgroup streams

    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    // ---- producer: the loading wavefronts ------------------------------------------------------
    // Load p of loading wavefront w fills block b = p * LW + w of the stage; blocks past the last
    // real one are padding and refetch it.
    const uint8_t* src[PER_LW];
    uint32_t step[PER_LW];                                    // bytes per stage along the source row
    const uint8_t* sbsrc[S::SB_BLOCKS];
    int p_tile = first, p_k = 0, p_tl = 0, p_kstart = 0;
    auto setup_src = [&](int tile) __attribute__((always_inline)) {
        const int t0 = (tile / tiles_o) * BT;
        const int o0 = (tile % tiles_o) * BO;
#pragma unroll
        for (int p = 0; p < PER_LW; ++p) {
            const int b = min(p * LW + wave_u, G::BLOCKS - 1);
            if (b < G::X_BLOCKS) {
                const int row = b * 8 + (lane >> 3);
                const int chunk = (lane & 7) ^ ((row >> 1) & 7);
                const int trow = min(t0 + row, a.tokens - 1);
                src[p] = reinterpret_cast<const uint8_t*>(a.X) + (size_t)trow * a.ldx + chunk * 16;
                step[p] = 128;
            } else if (b < G::X_BLOCKS + G::V_BLOCKS) {
                const int q = (b - G::X_BLOCKS) * 64 + lane;   // 16-byte slot index in the codes array
                const int row = min(q / (G::RV / 16), BO - 1);
                const int slot = q % (G::RV / 16);
                const int chunk = G::V_SWIZZLE ? (slot ^ ((row >> 1) & 7)) : slot;
                src[p] = a.vals + (size_t)(o0 + row) * a.vstride + chunk * 16;
                step[p] = G::RV;
            } else {
                const int q = (b - G::X_BLOCKS - G::V_BLOCKS) * 64 + lane;
                const int row = min(q / (G::RM / 16), BO - 1);
                src[p] = a.meta + (size_t)(o0 + row) * a.mstride + (q % (G::RM / 16)) * 16;
                step[p] = G::RM;
            }
        }
#pragma unroll
        for (int sb = 0; sb < S::SB_BLOCKS; ++sb) {
            const int f = (sb * 64 + lane) * 4;                // first of this lane's four floats
            const float* base = a.scales + o0;                 // lanes past both arrays refetch the first piece
            if (f < BO) base = a.scales + o0 + f;
            else if (f < 2 * BO && a.bias != nullptr) base = a.bias + o0 + (f - BO);
            sbsrc[sb] = reinterpret_cast<const uint8_t*>(base);
        }
        // Tiles walk K in rotated order (integer sums do not care), so that workgroups sharing
        // rows of X do not all miss on the same lines at the same moment.
        p_kstart = (int)(((unsigned)tile * 7u) % (unsigned)ns);
    };
    // Issues the next stage of the stream into ring slot `slot` and moves the producer cursor.
    auto issue_next = [&](int slot) __attribute__((always_inline)) {
        if (p_k == 0 && wave_u == 0) {
#pragma unroll
            for (int sb = 0; sb < S::SB_BLOCKS; ++sb)
                dma16(lds0 + S::SB_OFF + (p_tl % STAGES) * S::SB_BYTES + sb * 1024, sbsrc[sb]);
        }
        int k = p_kstart + p_k;
        if (k >= ns) k -= ns;
#pragma unroll
        for (int p = 0; p < PER_LW; ++p)
            dma16(lds0 + slot * STAGE + (p * LW + wave_u) * 1024, src[p] + (uint32_t)k * step[p]);
        if (++p_k == ns) {
            p_k = 0;
            ++p_tl;
            p_tile += gx;
            if (p_tile < last) setup_src(p_tile);
        }
    };

    // ---- consumer: fragments and accumulators ---------------------------------------------------
    v4i acc[FO][FT];
#pragma unroll
    for (int fo = 0; fo < FO; ++fo)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};

    const int xsw = (li >> 1) & 7;
    const int frag_x_lo = G::X_OFF + (wt * WT + li) * 128 + ((lg ^ xsw) * 16);
    const int frag_x_hi = G::X_OFF + (wt * WT + li) * 128 + (((lg + 4) ^ xsw) * 16);
    const int voff = lg * U::VBYTES;                           // byte offset of this lane's unit in the row
    const int vchunk = G::V_SWIZZLE ? ((voff >> 4) ^ xsw) : (voff >> 4);
    const int frag_v = G::V_OFF + (wo * WO + li) * G::RV + vchunk * 16 + (voff & 15);
    const int frag_m = G::M_OFF + (wo * WO + li) * G::RM + lg * U::MBYTES;

    struct Frags {
        v8i b[FT];
        typename U::Raw w[FO];
    };
    auto fetch = [&](int slot, Frags& f) __attribute__((always_inline)) {
        const uint8_t* base = smem + slot * STAGE;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const v4i lo = *reinterpret_cast<const v4i*>(base + frag_x_lo + ft * 16 * 128);
            const v4i hi = *reinterpret_cast<const v4i*>(base + frag_x_hi + ft * 16 * 128);
            f.b[ft] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
#pragma unroll
        for (int fo = 0; fo < FO; ++fo)
            f.w[fo] = U::load(base + frag_v + fo * 16 * G::RV, base + frag_m + fo * 16 * G::RM, 0);
    };
    auto mma = [&](const Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int fo = 0; fo < FO; ++fo) {
            v4i codes; int pos;
            U::decode(f.w[fo], codes, pos);
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(codes, f.b[ft], acc[fo][ft], pos, 0, 0);
        }
    };
    auto interleave = [&]() __attribute__((always_inline)) {
        // one MFMA, then one LDS read issued in its shadow
#pragma unroll
        for (int i = 0; i < FO * FT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
        }
    };

    // ---- epilogue of one tile: Eq. 4 with offset 0 on the product of two quantised operands -----
    // (ES is a compile-time constant so that the chunk arithmetic of the storing wavefronts folds
    // and their loop unrolls: all LDS reads first, then all stores.)
    int c_tile = first, c_k = 0, c_tl = 0;
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int t0 = (c_tile / tiles_o) * BT;
        const int o0 = (c_tile % tiles_o) * BO;
        const uint8_t* sbuf = smem + S::SB_OFF + (c_tl % STAGES) * S::SB_BYTES;
        const bool hb = a.bias != nullptr;
        uint8_t* stg = smem + S::ST_OFF;
        uint8_t* out = reinterpret_cast<uint8_t*>(a.out) + (size_t)o0 * ES;
        int_for<EP>([&](auto pass) __attribute__((always_inline)) {
            constexpr int P = decltype(pass)::value;
            constexpr int FPP = FT / EP;                        // fragment rows of a wavefront per pass
            wg_barrier();                                       // staging area is free (its last readers are done)
#pragma unroll
            for (int fo = 0; fo < FO; ++fo) {
                const int col = wo * WO + fo * 16 + 4 * lg;
                const float4 s4 = *reinterpret_cast<const float4*>(sbuf + col * 4);
                const float4 b4 = *reinterpret_cast<const float4*>(sbuf + (BO + col) * 4);
                const float sc[4] = {a.act_scale * s4.x, a.act_scale * s4.y, a.act_scale * s4.z, a.act_scale * s4.w};
                const float bs[4] = {hb ? b4.x : 0.f, hb ? b4.y : 0.f, hb ? b4.z : 0.f, hb ? b4.w : 0.f};
#pragma unroll
                for (int f = 0; f < FPP; ++f) {
                    const int srow = wt * (WT / EP) + f * 16 + li;
                    const v4i c = acc[fo][P * FPP + f];
                    float y[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) y[r] = (float)c[r] * sc[r] + bs[r];
                    uint8_t* dst = stg + srow * S::SROW_B + col * ES;
                    if constexpr (ES == 4) {
                        *reinterpret_cast<float4*>(dst) = make_float4(y[0], y[1], y[2], y[3]);
                    } else {
                        uint2 pk;
                        pk.x = pack_bf16x2(y[0], y[1]);
                        pk.y = pack_bf16x2(y[2], y[3]);
                        *reinterpret_cast<uint2*>(dst) = pk;
                    }
                }
            }
            wg_barrier_lds();                                   // staged rows complete
            if (!loader) {
                constexpr int CPR = BO * ES / 16;               // 16-byte chunks per staged row
                constexpr int CHUNKS = S::SROWS * CPR;
                constexpr int ITER = (CHUNKS + 64 * SW - 1) / (64 * SW);
                const int c0 = tid - 64 * LW;
                constexpr int BATCH = ITER < 6 ? ITER : 6;      // chunks a lane holds in registers at a time
#pragma unroll
                for (int i0 = 0; i0 < ITER; i0 += BATCH) {
                    v4i v[BATCH];
#pragma unroll
                    for (int i = 0; i < BATCH; ++i) {
                        const int c = min(c0 + (i0 + i) * 64 * SW, CHUNKS - 1);
                        const int srow = c / CPR, ch = c - srow * CPR;
                        v[i] = *reinterpret_cast<const v4i*>(stg + srow * S::SROW_B + ch * 16);
                    }
#pragma unroll
                    for (int i = 0; i < BATCH; ++i) {
                        const int c = c0 + (i0 + i) * 64 * SW;
                        const int srow = c / CPR, ch = c - srow * CPR;
                        // staged row -> row of the tile: wavefront row band, this pass's slice of it
                        const int band = srow / (WT / EP), in = srow - band * (WT / EP);
                        const int t = t0 + band * WT + P * (WT / EP) + in;
                        if (i0 + i < ITER && c < CHUNKS && t < a.tokens)
                            *reinterpret_cast<v4i*>(out + (size_t)t * a.ldo * ES + ch * 16) = v[i];
                    }
                }
            }
        });
#pragma unroll
        for (int fo = 0; fo < FO; ++fo)
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};
    };

    // ---- pipeline --------------------------------------------------------------------------------
    // Stream stage q sits in ring slot q % STAGES.  While stage q is multiplied, stages q+1 ..
    // q+AHEAD are landed or in flight, and the slot of stage q-1 is refilled.
    if (loader) {
        setup_src(p_tile);
#pragma unroll
        for (int j = 0; j <= AHEAD; ++j)
            if (j < total) issue_next(j % STAGES);
        if (total > AHEAD) wait_vm<AHEAD * PER_LW>();          // stage 0 landed; the AHEAD behind it may still fly
        else wait_vm<0>();
    }
    wg_barrier();

    Frags fr[2];
    fetch(0, fr[0]);
    int slot_c = 0;                             // ring slot of the stage being multiplied
    int slot_i = (AHEAD + 1) % STAGES;          // ring slot the next issue refills
    // Everything needed before the fragments of stage q+1 can be read.
    auto advance = [&](int q) __attribute__((always_inline)) {
        if (q + 1 < total) {
            if (loader) {
                // this wavefront's loads of stages q+1 .. min(q+AHEAD, total-1) are in flight, oldest first
                if (q + AHEAD < total) wait_vm<(AHEAD - 1) * PER_LW>();
                else wait_vm<0>();
            }
            wg_barrier();
            if (loader && q + 1 + AHEAD < total) issue_next(slot_i);
        }
        slot_c = (slot_c + 1 == STAGES) ? 0 : slot_c + 1;
        slot_i = (slot_i + 1 == STAGES) ? 0 : slot_i + 1;
    };
    auto tile_end = [&]() __attribute__((always_inline)) {
        if (++c_k == ns) {
            epilogue();
            c_k = 0;
            ++c_tl;
            c_tile += gx;
        }
    };
    // The fragment fetch is unconditional (after the last stage it re-reads an idle slot and the
    // values are dropped) so that the two register sets never merge across a branch.
    int q = 0;
    for (; q + 2 <= total; q += 2) {
        advance(q);
        mma(fr[0]);
        fetch(slot_c, fr[1]);
        interleave();
        tile_end();
        advance(q + 1);
        mma(fr[1]);
        fetch(slot_c, fr[0]);
        interleave();
        tile_end();
    }
    if (q < total) {
        advance(q);
        mma(fr[0]);
        tile_end();
    }
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int EP, int ES>
bool launch_stream_es(const GemmArgs& a, hipStream_t st)
{
    using S = StreamGeom<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, EP, ES>;
    if (a.O % BO != 0) return false;
    const int tiles_t = (a.tokens + BT - 1) / BT, tiles_o = a.O / BO;
    const int n_tiles = tiles_t * tiles_o;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return false;
        cus = prop.multiProcessorCount;
    }
    const int per_xcd = (n_tiles + 7) / 8;
    const int gx = per_xcd < cus / 8 ? per_xcd : cus / 8;     // workgroups per XCD: one per CU, fewer when tiles run out
    if (gx < 1) return false;
    auto kern = gemm_stream_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, EP, ES>;
    // Once per instantiation: raise the dynamic LDS limit (the attribute is sticky), and refuse a
    // build of the kernel that touches scratch memory, because scratch accesses are vector-memory
    // instructions the hand-counted waits of the loading wavefronts know nothing about.
    static int usable = -1;
    if (usable < 0) {
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kern)) != hipSuccess) return false;
        usable = (attr.localSizeBytes == 0) ? 1 : 0;
        if (usable && S::LDS > 64 * 1024)
            usable = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)S::LDS) == hipSuccess;
    }
    if (!usable) return false;
    hipLaunchKernelGGL(kern, dim3(8 * gx), dim3(64 * S::NW), S::LDS, st, a, tiles_o, n_tiles);
    return true;
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES, int EP>
bool launch_stream_tile(const GemmArgs& a, hipStream_t st)
{
    if (a.out_dtype == 1) return launch_stream_es<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, EP, 4>(a, st);
    return launch_stream_es<N, M, BITS, BT, BO, WAVES_T, WAVES_O, STAGES, EP, 2>(a, st);
}

template <int N, int M, int BITS>
bool launch_stream_pattern(const GemmArgs& a, hipStream_t st, int cfg)
{
    switch (cfg) {
        case 201: return launch_stream_tile<N, M, BITS, 128, 96, 4, 2, 3, 1>(a, st);
        case 202: return launch_stream_tile<N, M, BITS, 128, 96, 4, 2, 4, 1>(a, st);
        case 203: return launch_stream_tile<N, M, BITS, 128, 192, 4, 2, 3, 2>(a, st);
        case 204: return launch_stream_tile<N, M, BITS, 256, 96, 4, 2, 3, 4>(a, st);
        case 205: return launch_stream_tile<N, M, BITS, 128, 96, 2, 2, 4, 1>(a, st);
        case 206: return launch_stream_tile<N, M, BITS, 128, 128, 4, 2, 3, 1>(a, st);
        case 207: return launch_stream_tile<N, M, BITS, 128, 96, 4, 2, 5, 2>(a, st);
        case 208: return launch_stream_tile<N, M, BITS, 128, 96, 4, 2, 4, 2>(a, st);
        case 209: return launch_stream_tile<N, M, BITS, 256, 96, 4, 2, 3, 4>(a, st);
        default: return false;
    }
}

}  // namespace

// Returns true when it launched a kernel for this problem.
bool launch_gemm_stream(const GemmArgs& a, hipStream_t st, int cfg)
{
    const int esize = (a.out_dtype == 1) ? 4 : 2;
    if (a.acc != nullptr || (a.out_dtype != 1 && a.out_dtype != 2) || a.out == nullptr) return false;
    if (((size_t)a.ldo * esize) % 16 != 0 || (uintptr_t)a.out % 16 != 0) return false;
    if ((uintptr_t)a.scales % 16 != 0 || (uintptr_t)a.bias % 16 != 0 || (uintptr_t)a.meta % 16 != 0) return false;
    if (a.K % 128 != 0 || a.K < 128) return false;
#define NM_CASE(n, m, b) if (a.N == n && a.M == m && a.bits == b) return launch_stream_pattern<n, m, b>(a, st, cfg)
    NM_CASE(2, 4, 8);
#undef NM_CASE
    return false;
}

}  // namespace nm
