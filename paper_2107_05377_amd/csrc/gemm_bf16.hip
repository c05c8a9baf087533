// bfloat16 contraction on the gfx950 matrix cores:
//   C_g[M,N] = epi(A_g[M,K] * W_g[N,K]^T),  g = 0..G-1 in ONE launch (one problem per active task).
// Both operands are K-contiguous, which is the native MFMA operand order, so no transposition is
// needed anywhere.  Accumulation is float32 (v_mfma_f32_32x32x16_bf16).
//
// Tiling: a BM x BN output tile per workgroup, K consumed in slices of 64 through double-buffered
// LDS.  Global loads of slice k+1 are issued into registers before the MFMAs of slice k and written
// to the other LDS buffer afterwards, so one barrier per slice suffices.  LDS rows are 128 bytes
// (8 chunks of 16 bytes); chunk c of row r is stored at chunk c ^ (r & 7) so that the 16-byte
// fragment reads of 32 consecutive rows spread over all banks.
//
// Operand roles: the weight fragment is the first MFMA operand and the activation fragment the
// second, so a lane ends up with 4 consecutive output columns n of one output row m.  That makes
// bias loads, residual loads and stores 8- or 16-byte vectors along the row-major output.
//
// Workgroup -> tile mapping: consecutive workgroup ids go to different XCDs (8 of them, each with
// its own L2), so ids are first regrouped such that each XCD owns a contiguous range of tiles, and
// within a problem tiles are walked in bands of 8 row-tiles so that concurrently resident tiles
// share weight columns and activation rows in that XCD's L2.
#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int BK = 64;              // K slice (elements)
constexpr int ROW_BYTES = BK * 2;   // 128
constexpr int kXcds = 8;
constexpr int kBand = 8;            // row-tiles per raster band

template <int BM, int BN, int WAVES_M, int WAVES_N>
struct GemmCfg {
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TMI = WM / 32, TNI = WN / 32;
    static constexpr int A_CHUNKS = BM * 8 / NT, W_CHUNKS = BN * 8 / NT;
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BM % (WAVES_M * 32) == 0 && BN % (WAVES_N * 32) == 0, "wave tile must be a multiple of 32x32");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "tile rows must split evenly over threads");
};

__device__ inline int lds_chunk_off(int row, int chunk) { return row * ROW_BYTES + ((chunk ^ (row & 7)) << 4); }

template <int BM, int BN, int WAVES_M, int WAVES_N, bool OUT_F32>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_bf16_kernel(GemmGroup g, GemmShape s, int tiles_m,
                                                                          int tiles_n)
{
    using Cfg = GemmCfg<BM, BN, WAVES_M, WAVES_N>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- workgroup id -> (problem, row-tile, col-tile)
    const int total = s.G * tiles_m * tiles_n;
    int tile;
    {
        const int bid = blockIdx.x;
        const int x = bid % kXcds, i = bid / kXcds;
        const int q = total / kXcds, r = total % kXcds;
        tile = x * q + (x < r ? x : r) + i;
    }
    const int per_problem = tiles_m * tiles_n;
    const int grp = tile / per_problem;
    int t = tile - grp * per_problem;
    int tm, tn;
    {
        const int band_sz = kBand * tiles_n;
        const int band = t / band_sz;
        const int rows_in_band = min(kBand, tiles_m - band * kBand);
        const int tb = t - band * band_sz;
        tn = tb / rows_in_band;
        tm = band * kBand + tb % rows_in_band;
    }
    const int m0 = tm * BM, n0 = tn * BN;

    const __bf16* __restrict__ A = static_cast<const __bf16*>(g.A[grp]);
    const __bf16* __restrict__ W = static_cast<const __bf16*>(g.W[grp]);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * Cfg::WM, wn0 = (wave % WAVES_N) * Cfg::WN;
    const int l32 = lane & 31, half = lane >> 5;

    // ---- per-thread global source pointers and LDS destinations for the staging copies
    const __bf16* a_src[Cfg::A_CHUNKS];
    const __bf16* w_src[Cfg::W_CHUNKS];
    int a_dst[Cfg::A_CHUNKS], w_dst[Cfg::W_CHUNKS];
#pragma unroll
    for (int i = 0; i < Cfg::A_CHUNKS; ++i) {
        const int c = tid + i * Cfg::NT, row = c >> 3, ch = c & 7;
        const int gm = min(m0 + row, s.M - 1);
        a_src[i] = A + (size_t)gm * s.lda + ch * 8;
        a_dst[i] = lds_chunk_off(row, ch);
    }
#pragma unroll
    for (int i = 0; i < Cfg::W_CHUNKS; ++i) {
        const int c = tid + i * Cfg::NT, row = c >> 3, ch = c & 7;
        const int gn = min(n0 + row, s.N - 1);
        w_src[i] = W + (size_t)gn * s.K + ch * 8;
        w_dst[i] = BM * ROW_BYTES + lds_chunk_off(row, ch);
    }

    f32x16 acc[Cfg::TMI][Cfg::TNI];
#pragma unroll
    for (int i = 0; i < Cfg::TMI; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TNI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 a_reg[Cfg::A_CHUNKS], w_reg[Cfg::W_CHUNKS];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < Cfg::A_CHUNKS; ++i) a_reg[i] = *reinterpret_cast<const uint4*>(a_src[i] + k0);
#pragma unroll
        for (int i = 0; i < Cfg::W_CHUNKS; ++i) w_reg[i] = *reinterpret_cast<const uint4*>(w_src[i] + k0);
    };
    auto store_lds = [&](int buf) {
        unsigned char* base = lds + buf * Cfg::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::A_CHUNKS; ++i) *reinterpret_cast<uint4*>(base + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < Cfg::W_CHUNKS; ++i) *reinterpret_cast<uint4*>(base + w_dst[i]) = w_reg[i];
    };

    const int KT = s.K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_global((kt + 1) * BK);
        const unsigned char* sa = lds + (kt & 1) * Cfg::STAGE_BYTES;
        const unsigned char* sw = sa + BM * ROW_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[Cfg::TMI], wf[Cfg::TNI];
#pragma unroll
            for (int i = 0; i < Cfg::TMI; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(sa + lds_chunk_off(wm0 + i * 32 + l32, kk * 2 + half));
#pragma unroll
            for (int j = 0; j < Cfg::TNI; ++j)
                wf[j] = *reinterpret_cast<const bf16x8*>(sw + lds_chunk_off(wn0 + j * 32 + l32, kk * 2 + half));
#pragma unroll
            for (int i = 0; i < Cfg::TMI; ++i)
#pragma unroll
                for (int j = 0; j < Cfg::TNI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds, for tile (i,j): row m = ..+l32, columns n = ..+8*q+4*half+{0..3}, q=0..3
    const float* __restrict__ bias = g.bias[grp];
    const float* __restrict__ res = g.residual[grp];
    const int act = s.act;
#pragma unroll
    for (int i = 0; i < Cfg::TMI; ++i) {
        const int m = m0 + wm0 + i * 32 + l32;
        if (m >= s.M) continue;
#pragma unroll
        for (int j = 0; j < Cfg::TNI; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn0 + j * 32 + q * 8 + half * 4;
                if (n >= s.N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                if (bias) {
                    const float4 b = *reinterpret_cast<const float4*>(bias + n);
                    v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
                }
                if (act != ACT_NONE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], act);
                }
                if (res) {
                    const float4 r = *reinterpret_cast<const float4*>(res + (size_t)m * s.ldr + n);
                    v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w;
                }
                if constexpr (OUT_F32) {
                    float* C = static_cast<float*>(g.C[grp]);
                    *reinterpret_cast<float4*>(C + (size_t)m * s.ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    __bf16* C = static_cast<__bf16*>(g.C[grp]);
                    bf16x4 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                    *reinterpret_cast<bf16x4*>(C + (size_t)m * s.ldc + n) = o;
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_cfg(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    using Cfg = GemmCfg<BM, BN, WAVES_M, WAVES_N>;
    const int tiles_m = (s.M + BM - 1) / BM, tiles_n = (s.N + BN - 1) / BN;
    const int total = s.G * tiles_m * tiles_n;
    static bool attr_set[2] = {false, false};
    auto kf = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, true>;
    auto kb = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, false>;
    if (Cfg::LDS_BYTES > 64 * 1024) {
        const int which = s.out_f32 ? 0 : 1;
        if (!attr_set[which]) {
            hipError_t e = hipFuncSetAttribute(s.out_f32 ? (const void*)kf : (const void*)kb,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
            if (e != hipSuccess) return e;
            attr_set[which] = true;
        }
    }
    dim3 grid(total), block(Cfg::NT);
    if (s.out_f32) hipLaunchKernelGGL(kf, grid, block, Cfg::LDS_BYTES, stream, g, s, tiles_m, tiles_n);
    else hipLaunchKernelGGL(kb, grid, block, Cfg::LDS_BYTES, stream, g, s, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

int g_gemm_bf16_tile_override = 0;   // 0 = choose by shape; set through mt_debug_set_gemm_tile for tuning sweeps

hipError_t launch_gemm_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (s.G <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
    if (s.K % BK != 0 || s.K < BK || s.N % 4 != 0 || s.lda % 8 != 0 || s.ldc % 4 != 0 || s.ldr % 4 != 0 || s.G > kMaxGroup)
        return hipErrorInvalidValue;
    int sel = g_gemm_bf16_tile_override;
    if (sel == 0) {
        // Enough 256x128 tiles to fill 256 CUs at least ~3 times over -> larger tile; otherwise 128x128.
        const long t256 = (long)s.G * ((s.M + 255) / 256) * ((s.N + 127) / 128);
        sel = (t256 >= 768) ? 2 : 1;
    }
    switch (sel) {
        case 2: return launch_cfg<256, 128, 2, 2>(g, s, stream);
        case 3: return launch_cfg<256, 256, 2, 2>(g, s, stream);
        case 4: return launch_cfg<256, 256, 2, 4>(g, s, stream);
        case 5: return launch_cfg<128, 256, 2, 2>(g, s, stream);
        case 6: return launch_cfg<128, 128, 1, 4>(g, s, stream);
        default: return launch_cfg<128, 128, 2, 2>(g, s, stream);
    }
}

}  // namespace mt
