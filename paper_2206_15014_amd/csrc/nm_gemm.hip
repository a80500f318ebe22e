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

#include "nm_internal.h"

namespace nm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------------
// Weight units.  A unit is the slice of one packed weight row that covers 32 consecutive input
// columns: what one lane feeds to one sparse MFMA.
// ---------------------------------------------------------------------------------------------
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

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---------------------------------------------------------------------------------------------
// Sparse-MFMA GEMM.  One workgroup (4 wavefronts) computes a BT-token x BO-row output tile;
// K advances 128 input columns per step through two LDS stages:
//   X tile   BT rows x 128 bytes (row stride 144 to spread the fragment reads over the banks),
//   codes    BO rows x 64 bytes  (row stride 80),
//   positions BO rows x 16 bytes.
// Global loads of step k+1 are issued before the MFMAs of step k and parked in registers.
// Workgroups are numbered so that those sharing an XCD (blockIdx % 8) cover a contiguous token
// range: each XCD's L2 then holds one slice of X plus the (small) packed weight matrix.
// Requires K % 128 == 0, O % 4 == 0, 16-byte aligned X / ldx / values, ldo % 4 == 0.
// ---------------------------------------------------------------------------------------------
template <int BT, int BO>
struct TileGeom {
    static constexpr int XS = 144, WVS = 80, WMS = 16;
    static constexpr int STAGE = BT * XS + BO * WVS + BO * WMS;
};

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O>
__global__ void __launch_bounds__(256)
gemm_smfmac_kernel(const GemmArgs a, const int tiles_o, const int n_tiles)
{
    using U = Unit<N, M, BITS>;
    using G = TileGeom<BT, BO>;
    static_assert(WAVES_T * WAVES_O == 4, "four wavefronts per workgroup");
    constexpr int WT = BT / WAVES_T, WO = BO / WAVES_O;
    constexpr int FT = WT / 16, FO = WO / 16;
    constexpr int XCH = BT * 8 / 256;          // 16-byte X chunks per thread per step
    constexpr int WU = BO * 4 / 256;           // weight units per thread per step
    static_assert(XCH >= 1 && WU >= 1, "tile too small for 256 threads");

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

    // ---- global -> register staging -------------------------------------------------------
    const int8_t* xsrc[XCH];
#pragma unroll
    for (int r = 0; r < XCH; ++r) {
        const int c = tid + 256 * r;
        const int row = min(t0 + (c >> 3), a.tokens - 1);
        xsrc[r] = a.X + (size_t)row * a.ldx + (c & 7) * 16;
    }
    const uint8_t* wvsrc[WU];
    const uint8_t* wmsrc[WU];
#pragma unroll
    for (int r = 0; r < WU; ++r) {
        const int u = tid + 256 * r;
        const int row = min(o0 + (u >> 2), a.O - 1);
        wvsrc[r] = a.vals + (size_t)row * a.vstride;
        wmsrc[r] = a.meta + (size_t)row * a.mstride;
    }
    v4i xr[XCH];
    typename U::Raw wr[WU];

    auto gload = [&](int kt) {
#pragma unroll
        for (int r = 0; r < XCH; ++r) xr[r] = *reinterpret_cast<const v4i*>(xsrc[r] + (size_t)kt * 128);
#pragma unroll
        for (int r = 0; r < WU; ++r) wr[r] = U::load(wvsrc[r], wmsrc[r], kt * 4 + ((tid + 256 * r) & 3));
    };
    auto sstore = [&](int stage) {
        uint8_t* base = smem + stage * G::STAGE;
#pragma unroll
        for (int r = 0; r < XCH; ++r) {
            const int c = tid + 256 * r;
            *reinterpret_cast<v4i*>(base + (c >> 3) * G::XS + (c & 7) * 16) = xr[r];
        }
#pragma unroll
        for (int r = 0; r < WU; ++r) {
            const int u = tid + 256 * r;
            v4i codes; int pos;
            U::decode(wr[r], codes, pos);
            *reinterpret_cast<v4i*>(base + BT * G::XS + (u >> 2) * G::WVS + (u & 3) * 16) = codes;
            *reinterpret_cast<int*>(base + BT * G::XS + BO * G::WVS + (u >> 2) * G::WMS + (u & 3) * 4) = pos;
        }
    };

    v4i acc[FO][FT];
#pragma unroll
    for (int fo = 0; fo < FO; ++fo)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) acc[fo][ft] = v4i{0, 0, 0, 0};

    const int li = lane & 15, lg = lane >> 4;

    gload(0);
    sstore(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload(kt + 1);

        const uint8_t* base = smem + (kt & 1) * G::STAGE;
        const uint8_t* xs = base + (wt * WT + li) * G::XS + 16 * lg;
        const uint8_t* wv = base + BT * G::XS + (wo * WO + li) * G::WVS + 16 * lg;
        const uint8_t* wm = base + BT * G::XS + BO * G::WVS + (wo * WO + li) * G::WMS + 4 * lg;

        v8i bfr[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const v4i lo = *reinterpret_cast<const v4i*>(xs + ft * 16 * G::XS);
            const v4i hi = *reinterpret_cast<const v4i*>(xs + ft * 16 * G::XS + 64);
            bfr[ft] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
#pragma unroll
        for (int fo = 0; fo < FO; ++fo) {
            const v4i codes = *reinterpret_cast<const v4i*>(wv + fo * 16 * G::WVS);
            const int pos = *reinterpret_cast<const int*>(wm + fo * 16 * G::WMS);
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
                acc[fo][ft] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(codes, bfr[ft], acc[fo][ft], pos, 0, 0);
        }

        if (kt + 1 < nk) sstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: Eq. 4 with offset 0 on the product of two quantised operands --------------
#pragma unroll
    for (int fo = 0; fo < FO; ++fo) {
        const int o = o0 + wo * WO + fo * 16 + 4 * lg;
        if (o >= a.O) continue;
        const float4 sw = *reinterpret_cast<const float4*>(a.scales + o);
        const float sc[4] = {a.act_scale * sw.x, a.act_scale * sw.y, a.act_scale * sw.z, a.act_scale * sw.w};
        float bs[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.bias) {
            const float4 b = *reinterpret_cast<const float4*>(a.bias + o);
            bs[0] = b.x; bs[1] = b.y; bs[2] = b.z; bs[3] = b.w;
        }
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const int t = t0 + wt * WT + ft * 16 + li;
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
                } else {
                    uint2 p;
                    p.x = bf16_rne(y[0]) | (bf16_rne(y[1]) << 16);
                    p.y = bf16_rne(y[2]) | (bf16_rne(y[3]) << 16);
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + at) = p;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Any pattern, any shape, any alignment: one thread per output element, walking the metadata.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gemm_generic_kernel(const GemmArgs a)
{
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)a.tokens * a.O) return;
    const int t = (int)(id / a.O), o = (int)(id % a.O);
    const int ib = (a.M == 4) ? 2 : 4;
    const int kc = a.K / a.M * a.N;
    const uint8_t* vrow = a.vals + (size_t)o * a.vstride;
    const uint8_t* mrow = a.meta + (size_t)o * a.mstride;
    const int8_t* x = a.X + (size_t)t * a.ldx;
    int sum = 0;
    for (int e = 0; e < kc; ++e) {
        int q, off;
        if (a.bits == 8) q = (int8_t)vrow[e];
        else { int nib = (vrow[e >> 1] >> ((e & 1) * 4)) & 15; q = (nib ^ 8) - 8; }
        if (ib == 2) off = (mrow[e >> 2] >> ((e & 3) * 2)) & 3;
        else off = (mrow[e >> 1] >> ((e & 1) * 4)) & 15;
        sum += (int)x[(e / a.N) * a.M + off] * q;
    }
    const size_t at = (size_t)t * a.ldo + o;
    if (a.acc) a.acc[at] = sum;
    if (a.out_dtype != 0) {
        float y = (float)sum * (a.act_scale * a.scales[o]) + (a.bias ? a.bias[o] : 0.0f);
        if (a.out_dtype == 1) reinterpret_cast<float*>(a.out)[at] = y;
        else reinterpret_cast<uint16_t*>(a.out)[at] = (uint16_t)bf16_rne(y);
    }
}

template <int N, int M, int BITS, int BT, int BO, int WAVES_T, int WAVES_O>
void launch_tile(const GemmArgs& a, hipStream_t st)
{
    const int tiles_t = (a.tokens + BT - 1) / BT, tiles_o = (a.O + BO - 1) / BO;
    const int n_tiles = tiles_t * tiles_o;
    const int grid = 8 * ((n_tiles + 7) / 8);
    const size_t lds = 2 * (size_t)TileGeom<BT, BO>::STAGE;
    hipLaunchKernelGGL((gemm_smfmac_kernel<N, M, BITS, BT, BO, WAVES_T, WAVES_O>), dim3(grid), dim3(256), lds, st,
                       a, tiles_o, n_tiles);
}

template <int N, int M, int BITS>
void launch_pattern(const GemmArgs& a, hipStream_t st, int tile_cfg)
{
    // Enough workgroups to cover the 256 CUs decides the tile: big tiles reuse operands best,
    // small ones keep narrow layers (few output rows) from leaving CUs idle.
    const long long big = (long long)((a.tokens + 127) / 128) * ((a.O + 127) / 128);
    if (tile_cfg == 0) tile_cfg = (big >= 384) ? 1 : 2;
    switch (tile_cfg) {
        case 1: launch_tile<N, M, BITS, 128, 128, 2, 2>(a, st); break;
        case 2: launch_tile<N, M, BITS, 128, 64, 2, 2>(a, st); break;
        default: launch_tile<N, M, BITS, 64, 64, 2, 2>(a, st); break;
    }
}

}  // namespace

int launch_gemm(const GemmArgs& a, hipStream_t st)
{
    const bool out_ok = a.out_dtype == 0 || (uintptr_t)a.out % 16 == 0;
    const bool fast = a.N <= 2 && a.K % 128 == 0 && a.O % 4 == 0 && a.ldx % 16 == 0 && a.ldo % 4 == 0 &&
                      (uintptr_t)a.X % 16 == 0 && (uintptr_t)a.vals % 16 == 0 && (uintptr_t)a.meta % 4 == 0 &&
                      (uintptr_t)a.scales % 16 == 0 && (uintptr_t)a.bias % 16 == 0 && (uintptr_t)a.acc % 16 == 0 && out_ok;
    begin_launch();
    if (fast) {
        const char* env = getenv("NM_GEMM_TILE");   // tuning / test override of the tile choice
        const int tile_cfg = env ? atoi(env) : 0;
#define NM_CASE(n, m, b) else if (a.N == n && a.M == m && a.bits == b) launch_pattern<n, m, b>(a, st, tile_cfg)
        if (false) {}
        NM_CASE(2, 4, 8); NM_CASE(1, 4, 8); NM_CASE(2, 4, 4); NM_CASE(1, 4, 4);
        NM_CASE(1, 8, 8); NM_CASE(2, 8, 8); NM_CASE(1, 8, 4); NM_CASE(2, 8, 4);
#undef NM_CASE
    } else {
        const long long total = (long long)a.tokens * a.O;
        hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
    }
    return launch_status();
}

}  // namespace nm
