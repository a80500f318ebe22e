// nm_gemm, X-resident LDS-direct variant for gfx950: wide layers with a short reduction dimension
// (K <= 768: QKV and FFN-up of BERT-base).
//
// The ordinary kernel gives every workgroup one 256 x 192 output tile; at 4096 tokens that is one
// tile per CU, so a CU loads, multiplies and stores strictly one after the other and the output
// (the larger part of the layer's memory traffic) leaves while nothing else happens.  Here a
// workgroup keeps a 128-token tile of X whole in LDS (128 x K bytes, at most 96 KB, each slice
// loaded once, together with the first weight stages) and walks CT = 2 column tiles of 192
// against it.  Only packed weights are streamed for the second column tile (15 KB per 128-column
// slice instead of 31 KB), and the stores of the first column tile drain while the second one is
// multiplied.
//
// One in-order counter covers a wavefront's loads and stores alike, and the waits below are counted
// by hand, so the launcher only admits shapes for which every wavefront issues exactly the same
// memory instructions: whole token tiles, whole column tiles, 16-byte aligned output rows, and a
// kernel that keeps nothing in scratch.  Everything else goes to the other kernels.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "nm_gemm_common.h"

namespace nm {

namespace {

// KS = most 128-column slices of X the LDS area holds; CT = column tiles per workgroup.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int KS>
struct XresGeom {
    using G = DmaGeom<N, M, BITS, BT, BO, 1>;
    static constexpr int NW = WAVES_T * WAVES_O;
    static constexpr int STAGES = 3;                                    // weight ring
    static constexpr int CT = 2;
    static constexpr int X_SLICE = BT * 128;                            // one 128-column slice of the token tile
    static constexpr int XB = BT / 8;                                   // its 1 KB blocks (8 rows x 128 B)
    static constexpr int PX = XB / NW;                                  // X loads per wavefront and slice
    static constexpr int W_BLOCKS = G::V_BLOCKS + G::M_BLOCKS;          // one ring stage: codes, then index rows
    static constexpr int PW = (W_BLOCKS + NW - 1) / NW;                 // W loads per wavefront and stage
    static constexpr int STAGE = PW * NW * 1024;
    static constexpr int V_OFF = 0, M_OFF = G::V_BLOCKS * 1024;         // inside a stage
    static constexpr int RING_OFF = KS * X_SLICE;
    static constexpr int SB_OFF = RING_OFF + STAGES * STAGE;            // per column tile: 1 KB scales, 1 KB biases
    static constexpr int LDS = SB_OFF + CT * 2048;
    static_assert(XB % NW == 0, "every wavefront loads the same number of X blocks");
    static_assert(!G::PAIR_V && !G::PAIR_M, "whole 16-byte rows per stage only");
    static_assert(BO <= 256, "one direct load brings the scales of 256 columns");
    static_assert(LDS <= 160 * 1024, "exceeds the 160 KB of LDS of a CU");
};

// Grid: 8 * ceil(n_wgs / 8) workgroups; workgroup w -> unit (w % 8) * per_xcd + w / 8, unit u ->
// token tile u / groups, column tiles (u % groups) * CT ..: the workgroups that share a token tile
// sit on one XCD and share its L2.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int KS>
__global__ void __launch_bounds__(64 * WAVES_T * WAVES_O)
gemm_xres_kernel(const GemmArgs a, const int groups, const int n_wgs)
{
    using U = Unit<N, M, BITS>;
    using S = XresGeom<N, M, BITS, BT, BO, WAVES_T, WAVES_O, KS>;
    using G = typename S::G;
    constexpr int NW = S::NW, PX = S::PX, PW = S::PW, STAGE = S::STAGE, STAGES = S::STAGES, CT = S::CT;
    constexpr int WT = BT / WAVES_T, WO = BO / WAVES_O;
    constexpr int FT = WT / 16, FO = WO / 16;
    static_assert(WT % 16 == 0 && WO % 16 == 0, "wave tile must be whole 16x16 fragments");
    static_assert(FO % 2 == 0, "fragments pair up along the columns in the epilogue");
    static_assert((KS - 3) * PX + 3 * (PX + PW) + 1 < 64, "loads in flight must fit the counter");

    extern __shared__ __align__(1024) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wt = wave % WAVES_T, wo = wave / WAVES_T;
    const int li = lane & 15, lg = lane >> 4;

    const int per_xcd = (n_wgs + 7) >> 3;
    const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (unit >= n_wgs) return;                 // whole workgroup leaves before any barrier
    const int t0 = (unit / groups) * BT;
    const int o_first = (unit % groups) * CT * BO;
    const int ns = a.K >> 7;                   // 128-column slices, 3 <= ns <= KS (the host checks)
    const int total = CT * ns;                 // weight stages this workgroup streams

    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    // Scales and biases of both column tiles first: being the oldest loads of their wavefronts,
    // every later wait on the in-order counter covers them.  Lane l brings columns 4l .. 4l+3.
    static_assert(NW >= 2 * CT, "one wavefront per scale and bias block");
    if (wave_u < CT) {
        const uint32_t off = (uint32_t)min(o_first + wave_u * BO + 4 * lane, a.O - 4) * 4u;
        dma16s(lds0 + S::SB_OFF + wave_u * 2048, off, reinterpret_cast<const uint8_t*>(a.scales));
    } else if (wave_u < 2 * CT && a.bias != nullptr) {
        const uint32_t off = (uint32_t)min(o_first + (wave_u - CT) * BO + 4 * lane, a.O - 4) * 4u;
        dma16s(lds0 + S::SB_OFF + (wave_u - CT) * 2048 + 1024, off, reinterpret_cast<const uint8_t*>(a.bias));
    }

    // ---- sources ------------------------------------------------------------------------------
    // X: load p of wave w fills block p * NW + w of a slice (8 rows x 128 bytes, chunks swizzled).
    uint32_t xoff[PX];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        const int b = p * NW + wave_u;
        const int row = b * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        xoff[p] = (uint32_t)min(t0 + row, a.tokens - 1) * (uint32_t)a.ldx + chunk * 16;
    }
    // W: load p of wave w fills block p * NW + w of a stage; blocks past the last real one are
    // padding and refetch it.  Codes or index rows: decided by the wavefront, so base and step are scalars.
    uint32_t woff[PW];
    const uint8_t* wbase[PW];
    uint32_t wstep[PW], wjump[PW];             // bytes per slice; bytes from one column tile's rows to the next one's
#pragma unroll
    for (int p = 0; p < PW; ++p) {
        const int b = min(p * NW + wave_u, S::W_BLOCKS - 1);
        if (b < G::V_BLOCKS) {
            const int q = b * 64 + lane;                       // 16-byte slot index in the codes array
            const int row = min(q / (G::RV / 16), BO - 1);
            const int slot = q % (G::RV / 16);
            wbase[p] = a.vals;
            wstep[p] = G::RVS;
            wjump[p] = (uint32_t)BO * (uint32_t)a.vstride;
            woff[p] = (uint32_t)(o_first + row) * (uint32_t)a.vstride + (slot ^ G::v_xor(row)) * 16;
        } else {
            const int q = (b - G::V_BLOCKS) * 64 + lane;
            const int row = min(q / (G::RM / 16), BO - 1);
            wbase[p] = a.meta;
            wstep[p] = G::RMS;
            wjump[p] = (uint32_t)BO * (uint32_t)a.mstride;
            woff[p] = (uint32_t)(o_first + row) * (uint32_t)a.mstride + (q % (G::RM / 16)) * 16;
        }
    }
    const uint32_t lds_mine = lds0 + (uint32_t)wave_u * 1024u;
    int x_issue = 0;                           // next X slice to issue
    auto issue_x = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PX; ++p) {
            dma16s(lds_mine + (uint32_t)x_issue * S::X_SLICE + p * NW * 1024, xoff[p], reinterpret_cast<const uint8_t*>(a.X));
            xoff[p] += 128;
        }
        ++x_issue;
    };
    int w_k = 0;                               // slice of the next W stage to issue
    // Piece PART of PARTS of the next weight stage, into ring slot SLOT.
    auto issue_w = [&](auto slot, auto part, auto parts) __attribute__((always_inline)) {
        constexpr int SLOT = decltype(slot)::value, PART = decltype(part)::value, PARTS = decltype(parts)::value;
        constexpr int P0 = PART * PW / PARTS, P1 = (PART + 1) * PW / PARTS;
#pragma unroll
        for (int p = P0; p < P1; ++p) {
            dma16s(lds_mine + S::RING_OFF + SLOT * STAGE + p * NW * 1024, woff[p], wbase[p]);
            woff[p] += wstep[p];
        }
        if constexpr (PART == PARTS - 1) {
            if (++w_k == ns) {                 // on to the next column tile's rows
                w_k = 0;
#pragma unroll
                for (int p = 0; p < PW; ++p) woff[p] += wjump[p] - (uint32_t)ns * wstep[p];
            }
        }
    };
    using One = std::integral_constant<int, 1>;
    using Zero = std::integral_constant<int, 0>;

    v4i acc[FO][FT];
    auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int fo = 0; fo < FO; ++fo)
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};
    };
    clear_acc();

    // Fragment addresses (as in the ordinary kernel: fragment rows start at multiples of 16, so the
    // swizzle terms depend on the lane only).
    const int xsw = (li >> 1) & 7;
    const int frag_x_lo = (wt * WT + li) * 128 + ((lg ^ xsw) * 16);
    const int frag_x_hi = (wt * WT + li) * 128 + (((lg + 4) ^ xsw) * 16);
    const int voff_u = lg * U::VBYTES;
    const int frag_v = S::RING_OFF + S::V_OFF + (wo * WO + li) * G::RV + (((voff_u >> 4) ^ G::v_xor(li)) * 16) + (voff_u & 15);
    const int frag_m = S::RING_OFF + S::M_OFF + (wo * WO + li) * G::RM + lg * U::MBYTES;

    struct Frags {
        v8i b[FT];
        typename U::Raw w[FO];
    };
    Frags fr[2];
    auto read_b = [&](int k, auto ftc, v8i& dst) __attribute__((always_inline)) {
        constexpr int ft = decltype(ftc)::value;
        const uint8_t* base = smem + k * S::X_SLICE;
        const v4i lo = *reinterpret_cast<const v4i*>(base + frag_x_lo + ft * 16 * 128);
        const v4i hi = *reinterpret_cast<const v4i*>(base + frag_x_hi + ft * 16 * 128);
        dst = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };
    auto read_w = [&](auto slot, auto foc, typename U::Raw& dst) __attribute__((always_inline)) {
        constexpr int fo = decltype(foc)::value;
        const uint8_t* base = smem + decltype(slot)::value * STAGE;
        dst = U::load(base + frag_v + fo * 16 * G::RV, base + frag_m + fo * 16 * G::RM, 0);
    };

    // ---- epilogue of one column tile (Eq. 4 with offset 0; layout as in the ordinary kernel) --
    // NST store instructions per wavefront, every one of them issued by every wavefront.
    uint8_t* out = reinterpret_cast<uint8_t*>(a.out);
    const int row0 = t0 + wt * WT + li;
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    auto epilogue = [&](int c) __attribute__((always_inline)) {
        const int col0 = o_first + c * BO + wo * WO;
        const uint8_t* sb = smem + S::SB_OFF + c * 2048;
        int_for<FO / 2>([&](auto h) __attribute__((always_inline)) {
            constexpr int fo = 2 * decltype(h)::value;
            float4 sw[2], bw[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int cc = wo * WO + (fo + i) * 16 + 4 * lg;
                sw[i] = *reinterpret_cast<const float4*>(sb + cc * 4);
                bw[i] = a.bias ? *reinterpret_cast<const float4*>(sb + 1024 + cc * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            int_for<FT>([&](auto ftc) __attribute__((always_inline)) {
                constexpr int ft = decltype(ftc)::value;
                float y[2][4];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const v4i cv = acc[fo + i][ft];
                    y[i][0] = (float)cv[0] * (a.act_scale * sw[i].x) + bw[i].x;
                    y[i][1] = (float)cv[1] * (a.act_scale * sw[i].y) + bw[i].y;
                    y[i][2] = (float)cv[2] * (a.act_scale * sw[i].z) + bw[i].z;
                    y[i][3] = (float)cv[3] * (a.act_scale * sw[i].w) + bw[i].w;
                }
                const size_t row = (size_t)(row0 + ft * 16);
                if (a.out_dtype == 1) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        store16_through(out + (row * a.ldo + col0 + (fo + i) * 16 + 4 * lg) * 4,
                                        v4i{(int)__float_as_uint(y[i][0]), (int)__float_as_uint(y[i][1]),
                                            (int)__float_as_uint(y[i][2]), (int)__float_as_uint(y[i][3])});
                } else {
                    const v2u p = __builtin_amdgcn_permlane16_swap(pack_bf16x2(y[0][0], y[0][1]), pack_bf16x2(y[1][0], y[1][1]), false, false);
                    const v2u q = __builtin_amdgcn_permlane16_swap(pack_bf16x2(y[0][2], y[0][3]), pack_bf16x2(y[1][2], y[1][3]), false, false);
                    store16_through(out + (row * a.ldo + col0 + fo * 16 + (lg & 1) * 16 + (lg >> 1) * 8) * 2,
                                    v4i{(int)p[0], (int)q[0], (int)p[1], (int)q[1]});
                }
            });
        });
    };
    constexpr int NST_BF16 = FT * FO / 2, NST_F32 = FT * FO;
    static_assert(PW + NST_F32 < 64, "stores in flight must fit the counter");

    // ---- prologue -----------------------------------------------------------------------------
    // X slice k travels with weight stage k for k < 3; the remaining slices follow in one go, so
    // that every later issue is a weight stage and nothing else.
    int_for<STAGES>([&](auto q) __attribute__((always_inline)) {
        issue_x();
        issue_w(q, Zero{}, One{});
    });
    const int late = ns - STAGES;              // X slices issued behind the first three stages
    for (int k = STAGES; k < ns; ++k) issue_x();

    // Waits until at most `base + late * PX` of this wavefront's memory operations are outstanding.
    auto wait_late = [&](auto base) __attribute__((always_inline)) {
        constexpr int B = decltype(base)::value;
        static_assert(KS - STAGES <= 3, "one case per number of late slices");
        if (late <= 0) wait_vm<B>();
        else if (late == 1) wait_vm<B + PX>();
        else if (late == 2) wait_vm<B + 2 * PX>();
        else wait_vm<B + 3 * PX>();
    };
    wait_late(std::integral_constant<int, 2 * (PX + PW)>{});   // slice 0 and stage 0 landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int_for<FT>([&](auto ftc) __attribute__((always_inline)) { read_b(0, ftc, fr[0].b[decltype(ftc)::value]); });
    int_for<FO>([&](auto foc) __attribute__((always_inline)) { read_w(Zero{}, foc, fr[0].w[decltype(foc)::value]); });

    // ---- main loop ----------------------------------------------------------------------------
    // Stage q = c * ns + k (column tile c, slice k) sits in ring slot q % 3 and is multiplied in
    // step q.  By the barrier of step q every wavefront has read the last of stage q out of the
    // LDS (fragments are read a step ahead), so its slot is refilled with stage q + 3 right away:
    // two steps of latency from three slots.  The body covers 6 steps so that slots and fragment
    // sets are compile-time values.
    int c = 0, k = 0;
    const bool f32 = a.out_dtype == 1;
    for (int q0 = 0; q0 < total; q0 += 2 * STAGES) {
        int_for<2 * STAGES>([&](auto ss) __attribute__((always_inline)) {
            constexpr int SS = decltype(ss)::value;
            using Slot = std::integral_constant<int, SS % STAGES>;
            using Next = std::integral_constant<int, (SS + 1) % STAGES>;
            const int q = q0 + SS;
            if (q < total) {
                if (q + 1 < total) {
                    // Outstanding, oldest first, when stage q+1 must have landed:
                    //   q = 0:  slice 1 + stage 1 | slice 2 + stage 2, late slices
                    //   q = 1:  slice 2 + stage 2 | late slices, stage 3
                    //   first two steps of a later column tile: stage q+1 | stage q+2 and the
                    //   previous tile's stores (in either order)
                    //   otherwise: stage q+1 | stage q+2
                    if (q + 2 >= total) wait_vm<0>();
                    else if (q == 0) wait_late(std::integral_constant<int, PX + PW>{});
                    else if (q == 1) wait_late(std::integral_constant<int, PW>{});
                    else if (c > 0 && k < 2) {
                        if (f32) wait_vm<PW + NST_F32>();
                        else wait_vm<PW + NST_BF16>();
                    } else wait_vm<PW>();
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own reads of stage q done: its slot may be refilled
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
                const bool more = q + STAGES < total;
                const int kn = (k + 1 == ns) ? 0 : k + 1;    // slice of stage q+1
                int_for<FO>([&](auto g) __attribute__((always_inline)) {
                    constexpr int fo = decltype(g)::value;
                    // fragments of stage q+1 (after the last stage: a stale slot, dropped)
                    read_w(Next{}, g, fr[1 - SS % 2].w[fo]);
                    int_for<(fo + 1) * FT / FO - fo * FT / FO>([&](auto i) __attribute__((always_inline)) {
                        constexpr int ft = fo * FT / FO + decltype(i)::value;
                        read_b(kn, std::integral_constant<int, ft>{}, fr[1 - SS % 2].b[ft]);
                    });
                    v4i codes; int pos;
                    U::decode(fr[SS % 2].w[fo], codes, pos);
#pragma unroll
                    for (int ft = 0; ft < FT; ++ft)
                        acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(codes, fr[SS % 2].b[ft], acc[fo][ft], pos, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (more) issue_w(Slot{}, g, std::integral_constant<int, FO>{});
                    __builtin_amdgcn_sched_barrier(0);
                });
                if (k + 1 == ns) {
                    epilogue(c);
                    clear_acc();
                    ++c;
                    k = 0;
                } else {
                    ++k;
                }
            }
        });
    }
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int KS>
bool launch_xres_tile(const GemmArgs& a, hipStream_t st)
{
    using S = XresGeom<N, M, BITS, BT, BO, WAVES_T, WAVES_O, KS>;
    const int ns = a.K / 128;
    if (a.K % 128 != 0 || ns < S::STAGES || ns > KS) return false;
    if (a.tokens % BT != 0 || a.O % (S::CT * BO) != 0) return false;   // whole tiles only: every wavefront stores every fragment
    if ((unsigned long long)a.tokens * a.ldx >= (1ull << 32) || (unsigned long long)a.O * a.vstride >= (1ull << 32)) return false;
    const int groups = a.O / (S::CT * BO);
    const int n_wgs = (a.tokens / BT) * groups;
    auto kern = gemm_xres_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O, KS>;
    // Once per instantiation: raise the dynamic-LDS limit, and refuse a kernel that spills (scratch
    // accesses are memory instructions the hand-counted waits know nothing about).
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
    hipLaunchKernelGGL(kern, dim3(8 * ((n_wgs + 7) / 8)), dim3(64 * S::NW), S::LDS, st, a, groups, n_wgs);
    return true;
}

template <int N, int M, int BITS>
bool launch_xres_pattern(const GemmArgs& a, hipStream_t st, int cfg)
{
    using U = Unit<N, M, BITS>;
    if constexpr ((4 * U::VBYTES) % 16 != 0 || (4 * U::MBYTES) % 16 != 0) {
        return false;                                            // stage rows must be whole 16-byte pieces
    } else {
        switch (cfg) {
            case 301: return launch_xres_tile<N, M, BITS, 128, 192, 4, 2, 6>(a, st);   // wave tile 32 x 96
            case 302: return launch_xres_tile<N, M, BITS, 128, 192, 2, 2, 6>(a, st);   // 4 wavefronts, wave tile 64 x 96
            default: return false;
        }
    }
}

}  // namespace

// Returns true when it launched a kernel for this problem.
bool launch_gemm_xres(const GemmArgs& a, hipStream_t st, int cfg)
{
    const int esize = (a.out_dtype == 1) ? 4 : 2;
    if (a.acc != nullptr || (a.out_dtype != 1 && a.out_dtype != 2) || a.out == nullptr) return false;
    if (((size_t)a.ldo * esize) % 16 != 0 || (uintptr_t)a.out % 16 != 0) return false;
    if ((uintptr_t)a.scales % 16 != 0 || (uintptr_t)a.bias % 16 != 0) return false;
    if ((uintptr_t)a.vals % 16 != 0 || (uintptr_t)a.meta % 16 != 0 || a.vstride % 16 != 0 || a.mstride % 16 != 0) return false;
#define NM_CASE(n, m, b) if (a.N == n && a.M == m && a.bits == b) return launch_xres_pattern<n, m, b>(a, st, cfg)
    NM_CASE(2, 4, 8); NM_CASE(2, 4, 4); NM_CASE(2, 8, 8); NM_CASE(2, 8, 4);
#undef NM_CASE
    return false;
}

}  // namespace nm
