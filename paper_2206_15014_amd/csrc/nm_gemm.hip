// nm_gemm kernels for gfx950: the sparse integer linear layer of Sec. 5.3 with the
// dequantisation of Sec. 3.3 (Eq. 4, offset 0) fused behind it.
//
// Fast path (N <= 2): the weight operand goes to the structured-sparse integer MFMA
// v_smfmac_i32_16x16x128_i8, so products of pruned positions are never formed (Sec. 5.3:
// "only computing half the operations").  Any pattern with at most two kept entries per
// aligned 4-column subgroup is a legal operand of that instruction: 2:4 maps one to one,
// 1:4 / 1:8 / 2:8 are padded with explicit zeros while the tile is staged.  4-bit codes are
// sign-extended to int8 in registers first (Sec. 5.3: low-bit weights are widened to the
// activation type for the ALUs).
//
// Operand layout of v_smfmac_i32_16x16x128_i8 (A = 16 weight rows, B = 16 tokens, K = 128):
//   A  lane l: row l%16, the 16 kept codes of input columns [32*(l/16), 32*(l/16)+32) (two per
//      4-column subgroup, ascending), plus a dword whose bits [2e+1:2e] give the position of
//      code e inside its subgroup;
//   B  lane l: token l%16, bytes 0..15 = columns 16*(l/16)+0..15, bytes 16..31 = columns
//      64+16*(l/16)+0..15;
//   D  lane l, register r: weight row 4*(l/16)+r, token l%16.
// The 2:4 int8 packed format of include/nm.h is exactly the A layout, so that case is copied
// through untouched.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>


#include <type_traits>

#include "nm_internal.h"
#include "nm_gemm_common.h"

namespace nm {

namespace {

// ---------------------------------------------------------------------------------------------
// Sparse-MFMA GEMM.  One workgroup of WAVES_T x WAVES_O wavefronts computes a BT-token x BO-row
// output tile; K advances 128 input columns per step.
//
// Data path per step:  global --(16-byte loads, DEPTH steps ahead, parked in registers)-->
// registers --(decode of the weight units)--> LDS ring of STAGES stages --> MFMA fragments.
//   X tile    BT rows x 128 bytes (row stride 144 to spread the fragment reads over the banks),
//   codes     BO rows x 64 bytes  (row stride 80),
//   positions BO rows x 16 bytes.
// At these layer shapes the first touch of X comes from HBM, about a microsecond away, while
// one step's MFMAs take a fraction of that: the register ring keeps DEPTH steps of loads in
// flight per wavefront so the stream is bound by bandwidth rather than by one latency per step.
// With three LDS stages the stores of step k+2 are issued before the MFMAs of step k and only
// one barrier per step is needed; with two stages they follow the MFMAs.
//
// Workgroups are numbered so that those sharing an XCD (blockIdx % 8) cover a contiguous token
// range: each XCD's L2 then holds one slice of X plus the (small) packed weight matrix.
// Serves the row layout of the packed weights (the LDS-direct kernels read the tiled one).
// Requires K % 128 == 0, O % 4 == 0, 16-byte aligned X / ldx / values, ldo % 4 == 0.
// ---------------------------------------------------------------------------------------------
template <int BT, int BO>
struct TileGeom {
    static constexpr int XS = 144, WVS = 80, WMS = 16;
    static constexpr int STAGE = BT * XS + BO * WVS + BO * WMS;
};

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int DEPTH, int STAGES>
__global__ void __launch_bounds__(64 * WAVES_T * WAVES_O)
gemm_smfmac_kernel(const GemmArgs a, const int tiles_o, const int n_tiles)
{
    using U = Unit<N, M, BITS>;
    using G = TileGeom<BT, BO>;
    constexpr int NT = 64 * WAVES_T * WAVES_O;
    constexpr int WT = BT / WAVES_T, WO = BO / WAVES_O;
    constexpr int FT = WT / 16, FO = WO / 16;
    static_assert(WT % 16 == 0 && WO % 16 == 0, "wave tile must be whole 16x16 fragments");
    static_assert(STAGES == 2 || STAGES == 3, "two or three LDS stages");
    constexpr int XCH = (BT * 8 + NT - 1) / NT;   // 16-byte X chunks per thread per step
    constexpr int WU = (BO * 4 + NT - 1) / NT;    // weight units per thread per step
    constexpr bool XFULL = (BT * 8) % NT == 0, WFULL = (BO * 4) % NT == 0;

    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wt = wave % WAVES_T, wo = wave / WAVES_T;

    const int per_xcd = (n_tiles + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= n_tiles) return;               // whole workgroup leaves before any barrier
    const int t0 = (tile / tiles_o) * BT;
    const int o0 = (tile % tiles_o) * BO;

    const int nk = a.K >> 7;

    // ---- global -> register ring ------------------------------------------------------------
    const int8_t* xsrc[XCH];
#pragma unroll
    for (int r = 0; r < XCH; ++r) {
        const int c = min(tid + NT * r, BT * 8 - 1);
        const int row = min(t0 + (c >> 3), a.tokens - 1);
        xsrc[r] = a.X + (size_t)row * a.ldx + (c & 7) * 16;
    }
    const uint8_t* wvsrc[WU];
    const uint8_t* wmsrc[WU];
#pragma unroll
    for (int r = 0; r < WU; ++r) {
        const int u = min(tid + NT * r, BO * 4 - 1);
        const int row = min(o0 + (u >> 2), a.O - 1);
        wvsrc[r] = a.vals + (size_t)row * a.pv.stride + (u & 3) * U::VBYTES;
        wmsrc[r] = a.meta + (size_t)row * a.pm.stride + (u & 3) * U::MBYTES;
    }
    v4i xr[DEPTH][XCH];
    typename U::Raw wr[DEPTH][WU];

    auto gload = [&](int kt, auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
#pragma unroll
        for (int r = 0; r < XCH; ++r) xr[slot][r] = *reinterpret_cast<const v4i*>(xsrc[r] + (size_t)kt * 128);
#pragma unroll
        for (int r = 0; r < WU; ++r) wr[slot][r] = U::load(wvsrc[r], wmsrc[r], kt * 4);
    };
    auto sstore = [&](int stage, auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        uint8_t* base = smem + stage * G::STAGE;
#pragma unroll
        for (int r = 0; r < XCH; ++r) {
            const int c = tid + NT * r;
            if (XFULL || c < BT * 8)
                *reinterpret_cast<v4i*>(base + (c >> 3) * G::XS + (c & 7) * 16) = xr[slot][r];
        }
#pragma unroll
        for (int r = 0; r < WU; ++r) {
            const int u = tid + NT * r;
            if (WFULL || u < BO * 4) {
                v4i codes; int pos;
                U::decode(wr[slot][r], codes, pos);
                *reinterpret_cast<v4i*>(base + BT * G::XS + (u >> 2) * G::WVS + (u & 3) * 16) = codes;
                *reinterpret_cast<int*>(base + BT * G::XS + BO * G::WVS + (u >> 2) * G::WMS + (u & 3) * 4) = pos;
            }
        }
    };

    v4i acc[FO][FT];
#pragma unroll
    for (int fo = 0; fo < FO; ++fo)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};

    const int li = lane & 15, lg = lane >> 4;
    const int frag_x = (wt * WT + li) * G::XS + 16 * lg;
    const int frag_v = BT * G::XS + (wo * WO + li) * G::WVS + 16 * lg;
    const int frag_p = BT * G::XS + BO * G::WVS + (wo * WO + li) * G::WMS + 4 * lg;

    auto compute = [&](int stage) {
        const uint8_t* base = smem + stage * G::STAGE;
        v8i bfr[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const v4i lo = *reinterpret_cast<const v4i*>(base + frag_x + ft * 16 * G::XS);
            const v4i hi = *reinterpret_cast<const v4i*>(base + frag_x + ft * 16 * G::XS + 64);
            bfr[ft] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
#pragma unroll
        for (int fo = 0; fo < FO; ++fo) {
            const v4i codes = *reinterpret_cast<const v4i*>(base + frag_v + fo * 16 * G::WVS);
            const int pos = *reinterpret_cast<const int*>(base + frag_p + fo * 16 * G::WMS);
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(codes, bfr[ft], acc[fo][ft], pos, 0, 0);
        }
    };

    // Register slot of step j is j % DEPTH; LDS stage of step j is j % STAGES.  The host only
    // picks a DEPTH that divides the step count, and loads past the last step re-read the last
    // step (in bounds, never consumed): the loop body is then free of data-dependent branches,
    // which lets the compiler count exactly how many younger loads may stay in flight at each
    // wait instead of draining the queue.
    constexpr int LEAD = STAGES - 1;           // steps resident in LDS ahead of the one being computed
    const int last = nk - 1;
    int_for<DEPTH>([&](auto d) { gload(min((int)d.value, last), d); });
    int_for<LEAD>([&](auto j) {
        using Slot = std::integral_constant<int, j.value % DEPTH>;
        sstore(j.value % STAGES, Slot{});
        gload(min((int)j.value + DEPTH, last), Slot{});
    });
    __syncthreads();

    int stage_c = 0;                            // kt % STAGES
    int stage_s = LEAD % STAGES;                // (kt + LEAD) % STAGES
    for (int kt0 = 0; kt0 < nk; kt0 += DEPTH) {
        int_for<DEPTH>([&](auto d) {
            const int kt = kt0 + d.value;
            using Slot = std::integral_constant<int, (d.value + LEAD) % DEPTH>;
            if constexpr (STAGES == 3) {
                sstore(stage_s, Slot{});
                gload(min(kt + LEAD + DEPTH, last), Slot{});
                compute(stage_c);
            } else {
                compute(stage_c);
                sstore(stage_s, Slot{});
                gload(min(kt + LEAD + DEPTH, last), Slot{});
            }
            __syncthreads();
            stage_c = (stage_c + 1 == STAGES) ? 0 : stage_c + 1;
            stage_s = (stage_s + 1 == STAGES) ? 0 : stage_s + 1;
        });
    }

    store_tile<FO, FT>(a, acc, o0 + wo * WO, t0 + wt * WT, li, lg);
}

// ---------------------------------------------------------------------------------------------
// Any pattern, any shape, any alignment, either layout: one thread per output element, walking
// the metadata.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gemm_generic_kernel(const GemmArgs a)
{
    const long long id_raw = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)a.tokens * a.O;
    const bool live = id_raw < total;          // threads past the end recompute the last output and store nothing
    const long long id = live ? id_raw : total - 1;
    const int t = (int)(id / a.O), o = (int)(id % a.O);
    const int ib = (a.N >= a.M) ? 0 : (a.M == 4) ? 2 : 4;
    const int kc = a.K / a.M * a.N;
    const int8_t* x = a.X + (size_t)t * a.ldx;
    int sum = 0;
    for (int e = 0; e < kc; ++e) {
        int q, off;
        if (a.bits == 8) q = (int8_t)a.vals[a.pv.at((uint32_t)o, (uint32_t)e)];
        else { int nib = (a.vals[a.pv.at((uint32_t)o, (uint32_t)e >> 1)] >> ((e & 1) * 4)) & 15; q = (nib ^ 8) - 8; }
        if (ib == 0) off = e % a.N;
        else if (ib == 2) off = (a.meta[a.pm.at((uint32_t)o, (uint32_t)e >> 2)] >> ((e & 3) * 2)) & 3;
        else off = (a.meta[a.pm.at((uint32_t)o, (uint32_t)e >> 1)] >> ((e & 1) * 4)) & 15;
        sum += (int)x[(e / a.N) * a.M + off] * q;
    }
    const size_t at = (size_t)t * a.ldo + o;
    const float s_act = act_scale_of(a);
    if (a.out_dtype == 3) {                    // requantised output: every lane takes part in the reduction of max |y|
        const float s_out = out_scale_of(a);
        float g[4] = {0.f, 0.f, 0.f, 0.f}, h[4] = {0.f, 0.f, 0.f, 0.f};
        requant_column(s_act, a.scales[o], a.bias ? a.bias[o] : 0.0f, s_out, g[0], h[0]);
        float m = 0.0f;
        const uint32_t q = requant4(v4i{sum, 0, 0, 0}, g, h, m);
        if (live) reinterpret_cast<uint8_t*>(a.out)[at] = (uint8_t)q;
        absmax_commit(m, s_out, a.absmax);
        return;
    }
    if (!live) return;
    if (a.acc) a.acc[at] = sum;
    if (a.out_dtype != 0) {
        float y = (float)sum * (s_act * a.scales[o]) + (a.bias ? a.bias[o] : 0.0f);
        if (a.out_dtype == 1) reinterpret_cast<float*>(a.out)[at] = y;
        else reinterpret_cast<uint16_t*>(a.out)[at] = (uint16_t)pack_bf16x2(y, 0.0f);
    }
}

// Register-resident loop of the sparse MFMA (measurement hook, see nm_test_hooks.h).
__global__ void __launch_bounds__(256)
smfmac_probe_kernel(int iters, unsigned long long* counters)
{
    const int lane = threadIdx.x & 63;
    v4i a = v4i{lane, lane + 1, lane + 2, lane + 3};
    v8i b = v8i{lane, 1, 2, 3, 4, 5, 6, lane};
    v4i acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = v4i{k, 0, 0, 0};
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a, b, acc[k], 0x44444444, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    int sum = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) sum += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        counters[0] = (unsigned long long)(c1 - c0);
        counters[1] = (unsigned long long)(w1 - w0);
    }
    if (sum == 0x7fffffff) counters[2] = (unsigned long long)sum;     // keeps the loop alive; never true in practice
}

// Scale of 8-bit activations from their largest magnitude (the rule of Sec. 3.3.1 at 8 bits).
__global__ void absmax_to_scale_kernel(float* absmax, float* scale, int reset)
{
    const float m = *absmax;
    *scale = (m == 0.0f) ? 1.0f : __fdiv_rn(m, 127.0f);
    if (reset) *absmax = 0.0f;
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int DEPTH, int STAGES>
void launch_tile(const GemmArgs& a, hipStream_t st)
{
    if constexpr (DEPTH > 1) {
        if ((a.K / 128) % DEPTH != 0) {         // the kernel's ring needs a whole number of rounds
            launch_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, 1, STAGES>(a, st);
            return;
        }
    }
    const int tiles_t = (a.tokens + BT - 1) / BT, tiles_o = (a.O + BO - 1) / BO;
    const int n_tiles = tiles_t * tiles_o;
    const int grid = 8 * ((n_tiles + 7) / 8);
    const size_t lds = STAGES * (size_t)TileGeom<BT, BO>::STAGE;
    auto kern = gemm_smfmac_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O, DEPTH, STAGES>;
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> raised{0};   // per instantiation
        raise_lds_limit(reinterpret_cast<const void*>(kern), lds, raised);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WAVES_T * WAVES_O), lds, st, a, tiles_o, n_tiles);
}

// Ring depth: the deepest of 4, 3, 2, 1 that divides the number of 128-column steps.
template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O, int STAGES>
void launch_depth(const GemmArgs& a, hipStream_t st)
{
    const int nk = a.K / 128;
    if (nk % 4 == 0) launch_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, 4, STAGES>(a, st);
    else if (nk % 3 == 0) launch_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, 3, STAGES>(a, st);
    else if (nk % 2 == 0) launch_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, 2, STAGES>(a, st);
    else launch_tile<N, M, BITS, BT, BO, WAVES_T, WAVES_O, 1, STAGES>(a, st);
}

template <int N, int M, int BITS>
void launch_pattern(const GemmArgs& a, hipStream_t st, int tile_cfg)
{
    // Enough workgroups to cover the 256 CUs decides the tile: big tiles reuse operands best,
    // small ones keep narrow layers (few output rows) from leaving CUs idle.
    const long long big = (long long)((a.tokens + 127) / 128) * ((a.O + 127) / 128);
    if (tile_cfg < 1 || tile_cfg > 3) tile_cfg = (big >= 384) ? 1 : 2;
    note_gemm_tile(tile_cfg);
    switch (tile_cfg) {
        case 1: launch_depth<N, M, BITS, 128, 128, 2, 2, 2>(a, st); break;
        case 2: launch_depth<N, M, BITS, 128, 64, 2, 2, 2>(a, st); break;
        default: launch_depth<N, M, BITS, 64, 64, 2, 2, 2>(a, st); break;
    }
}

}  // namespace

bool launch_gemm_dma_set0(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set1(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set2(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set3(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set4(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set5(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set6(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set7(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set8(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set9(const GemmArgs* items, int count, hipStream_t st, int cfg);
bool launch_gemm_dma_set10(const GemmArgs* items, int count, hipStream_t st, int cfg);

bool launch_gemm_dma(const GemmArgs* items, int count, hipStream_t st, int cfg)
{
    return launch_gemm_dma_set0(items, count, st, cfg) || launch_gemm_dma_set1(items, count, st, cfg) ||
           launch_gemm_dma_set2(items, count, st, cfg) || launch_gemm_dma_set3(items, count, st, cfg) ||
           launch_gemm_dma_set4(items, count, st, cfg) || launch_gemm_dma_set5(items, count, st, cfg) ||
           launch_gemm_dma_set6(items, count, st, cfg) || launch_gemm_dma_set7(items, count, st, cfg) ||
           launch_gemm_dma_set8(items, count, st, cfg) || launch_gemm_dma_set9(items, count, st, cfg) ||
           launch_gemm_dma_set10(items, count, st, cfg);
}

int launch_smfmac_probe(int blocks, int iters, unsigned long long* counters, hipStream_t st)
{
    begin_launch();
    hipLaunchKernelGGL(smfmac_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, st, iters, counters);
    return launch_status();
}

int launch_absmax_to_scale(float* absmax, float* scale, int reset, hipStream_t st)
{
    begin_launch();
    hipLaunchKernelGGL(absmax_to_scale_kernel, dim3(1), dim3(1), 0, st, absmax, scale, reset);
    return launch_status();
}

namespace {

// What the matrix-core kernels ask of a call beyond the ABI's own requirements.
bool fast_path_ok(const GemmArgs& a)
{
    const bool out_ok = a.out_dtype == 0 || (uintptr_t)a.out % 16 == 0;   // (int8 codes: rows are then whole dwords, ldo % 4 == 0)
    return a.K % 128 == 0 && a.O % 4 == 0 && a.ldx % 16 == 0 && a.ldo % 4 == 0 &&
           (uintptr_t)a.X % 16 == 0 && (uintptr_t)a.vals % 16 == 0 && (uintptr_t)a.meta % 16 == 0 &&
           (uintptr_t)a.scales % 16 == 0 && (uintptr_t)a.bias % 16 == 0 && (uintptr_t)a.acc % 16 == 0 && out_ok;
}

}  // namespace

int launch_gemm_batch(const GemmArgs* items, int count, hipStream_t st)
{
    bool together = count > 1;
    for (int i = 0; i < count && together; ++i) together = fast_path_ok(items[i]) && items[i].pv.tiled;
    if (together) {
        begin_launch();
        const int tile_cfg = forced_gemm_tile();
        if (launch_gemm_dma(items, count, st, tile_cfg >= 100 ? tile_cfg : 0)) return launch_status();
    }
    for (int i = 0; i < count; ++i) {
        const int rc = launch_gemm(items[i], st);
        if (rc) return rc;
    }
    return 0;
}

int launch_gemm(const GemmArgs& a, hipStream_t st)
{
    const bool fast = fast_path_ok(a);
    begin_launch();
    const int tile_cfg = forced_gemm_tile();    // 0 unless a test forces a variant
    // Tiled layout: the LDS-direct kernels (tile_cfg 0 = their own choice, >= 100 = a forced variant).
    if (fast && a.pv.tiled && launch_gemm_dma(&a, 1, st, tile_cfg >= 100 ? tile_cfg : 0)) return launch_status();
    // Row layout, at most two kept per group: the register-staged kernel (tile_cfg 1 .. 3 force its shapes).
    if (fast && !a.pv.tiled && a.N <= 2) {
#define NM_CASE(n, m, b) else if (a.N == n && a.M == m && a.bits == b) launch_pattern<n, m, b>(a, st, tile_cfg)
        if (false) {}
        NM_CASE(2, 4, 8); NM_CASE(1, 4, 8); NM_CASE(2, 4, 4); NM_CASE(1, 4, 4);
        NM_CASE(1, 8, 8); NM_CASE(2, 8, 8); NM_CASE(1, 8, 4); NM_CASE(2, 8, 4);
#undef NM_CASE
        return launch_status();
    }
    const long long total = (long long)a.tokens * a.O;
    hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
    note_gemm_tile(-1);
    return launch_status();
}

}  // namespace nm
