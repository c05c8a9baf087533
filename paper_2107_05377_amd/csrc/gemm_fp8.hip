// FP8 (OCP E4M3) contraction on the gfx950 matrix cores, the reduced-precision variant of the two feed-forward
// contractions:   C_g[M,N] = epi(scale_g * (A_g[M,K] * W_g[N,K]^T)),  A and W one byte per element, K contiguous,
// float32 accumulation (v_mfma_f32_32x32x64_f8f6f4: 64 K elements per instruction, twice the bf16 rate).
// scale_g undoes the power-of-two scaling the weights were stored with.
//
// Same persistent organisation as gemm_bf16_persist.hip: one workgroup per compute unit walks a list of 256 x 256
// tiles, the ring of K slices (global_load_lds, XOR-swizzled 16-byte chunks) never drains between tiles, the
// epilogue parks accumulators in an LDS region of its own.  A K slice is 64 elements = 64 bytes per row, so the
// ring has byte for byte the layout of the bf16 kernel's 32-wide slices.  What differs is the inner pipeline: a
// slice is ONE matrix instruction per 32x32 block, so there are no K steps to pipeline fragment reads across.
// Instead slice kt is multiplied out of registers while the fragments of slice kt+1 are read: the 4 activation
// fragments are reloaded in place, each right after the two instructions that use it, the 2 weight fragments into a
// second set.  Since a slice is in registers before it is multiplied, its ring stage is free one slice earlier than
// in the bf16 kernel, and the refill of slice kt+STAGES is issued right after the barrier of slice kt.
#include <algorithm>

#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int kFXcds = 8;
constexpr int kFBand = 8;

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8;
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int N>
__device__ __forceinline__ void f_wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void f_wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int ACT>
__device__ __forceinline__ float f_act(float v)
{
    if constexpr (ACT == ACT_GELU_ERF) return gelu_erf_fast(v);
    else if constexpr (ACT == ACT_GELU_TANH) return gelu_tanh(v);
    else return v;
}

constexpr int F_BM = 256, F_BN = 256, F_WAVES_M = 2, F_WAVES_N = 4, F_NW = 8;
constexpr int F_ROW_BYTES = 64, F_CH = 4, F_RPI = 16, F_KEY_SHIFT = 2, F_BK = 64;
constexpr int F_WM = F_BM / F_WAVES_M, F_WN = F_BN / F_WAVES_N, F_TMI = F_WM / 32, F_TNI = F_WN / 32;
constexpr int F_A_LOADS = F_BM / F_RPI / F_NW, F_W_LOADS = F_BN / F_RPI / F_NW, F_LPS = F_A_LOADS + F_W_LOADS;
constexpr int F_STAGE_BYTES = (F_BM + F_BN) * F_ROW_BYTES;
constexpr int F_PARK_ROWB = F_WN * 4, F_PARK_BYTES = 32 * F_PARK_ROWB;

struct FTile {
    const unsigned char* A;
    const unsigned char* W;
    uint32_t off[F_LPS];
    int grp, m0, n0;
};

// OUT: 0 bfloat16, 1 float32 (+ optional residual), 2 E4M3 (the value times s.out_scale)
template <int STAGES, int OUT, int ACT>
__global__ __launch_bounds__(F_NW * 64, 1) void gemm_fp8_kernel(GemmGroup g, GemmShape s, int tiles_n)
{
    constexpr int RING_BYTES = STAGES * F_STAGE_BYTES;
    static_assert(STAGES >= 2 && RING_BYTES + F_NW * F_PARK_BYTES <= 160 * 1024, "LDS");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int M = s.d_M ? min(s.M, *s.d_M) : s.M;
    const int tiles_m = (M + F_BM - 1) / F_BM;
    const int per_problem = tiles_m * tiles_n;
    const int total = s.G * per_problem;
    // XCD x owns tiles [lo, lo + cnt), its workgroups stride through them (a launch of fewer workgroups than XCDs is one range)
    const int xcds = (int)gridDim.x >= kFXcds ? kFXcds : 1;
    const int xcd = blockIdx.x % xcds, wi = blockIdx.x / xcds;
    const int wg_x = ((int)gridDim.x - xcd + xcds - 1) / xcds;
    const int q = total / xcds, r = total % xcds;
    const int lo = xcd * q + min(xcd, r), cnt = q + (xcd < r ? 1 : 0);
    if (wi >= cnt) return;                                                   // uniform over the workgroup
    const int n_mine = (cnt - wi + wg_x - 1) / wg_x;

    const int KT = s.K / F_BK;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / F_WAVES_N) * F_WM, wn0 = (wave % F_WAVES_N) * F_WN;
    const int l32 = lane & 31, half = lane >> 5;
    const uint32_t lda_b = (uint32_t)s.lda, ldw_b = (uint32_t)(s.ldw ? s.ldw : s.K);

    int ld_row[F_LPS], ld_chunk[F_LPS];
#pragma unroll
    for (int i = 0; i < F_LPS; ++i) {
        const bool isA = i < F_A_LOADS;
        ld_row[i] = (wave + (isA ? i : i - F_A_LOADS) * F_NW) * F_RPI + lane / F_CH;
        ld_chunk[i] = ((lane % F_CH) ^ ((ld_row[i] >> F_KEY_SHIFT) & (F_CH - 1))) * 16;
    }
    auto locate = [&](int j, FTile& t) {
        const int tile = lo + wi + j * wg_x;
        t.grp = tile / per_problem;
        const int tt = tile - t.grp * per_problem;
        const int band_sz = kFBand * tiles_n;
        const int band = tt / band_sz;
        const int rows_in_band = min(kFBand, tiles_m - band * kFBand);
        const int tb = tt - band * band_sz;
        const int tn = tb / rows_in_band;
        const int tm = band * kFBand + tb % rows_in_band;
        t.m0 = tm * F_BM;
        t.n0 = tn * F_BN;
        t.A = static_cast<const unsigned char*>(g.A[t.grp]);
        t.W = static_cast<const unsigned char*>(g.W[t.grp]);
#pragma unroll
        for (int i = 0; i < F_LPS; ++i) {
            if (i < F_A_LOADS) t.off[i] = (uint32_t)min(t.m0 + ld_row[i], M - 1) * lda_b + ld_chunk[i];
            else t.off[i] = (uint32_t)min(t.n0 + ld_row[i], s.N - 1) * ldw_b + ld_chunk[i];
        }
    };
    // A lane's fragment of a 32-row block: K bytes [32 half, 32 half + 32) of row l32 = chunks 2 half and 2 half + 1,
    // which sit in slots (chunk ^ key(row)): the second one is the first with bit 4 of the byte address flipped.
    const int f_off = l32 * F_ROW_BYTES + (((2 * half) ^ ((l32 >> F_KEY_SHIFT) & (F_CH - 1))) << 4);
    const int fa_off = wm0 * F_ROW_BYTES + f_off;
    const int fw_off = (F_BM + wn0) * F_ROW_BYTES + f_off;

    FTile cur, nxt;
    locate(0, cur);

#define MT_F_ISSUE(t_, slice_, stage_)                                                                              \
    do {                                                                                                            \
        const unsigned char* a_k = (t_).A + (size_t)(slice_) * F_ROW_BYTES;                                         \
        const unsigned char* w_k = (t_).W + (size_t)(slice_) * F_ROW_BYTES;                                         \
        unsigned char* sbase = lds + (stage_) * F_STAGE_BYTES;                                                      \
        _Pragma("unroll") for (int i_ = 0; i_ < F_LPS; ++i_) {                                                      \
            if (i_ < F_A_LOADS)                                                                                     \
                __builtin_amdgcn_global_load_lds((gptr_t)(a_k + (t_).off[i_]),                                      \
                                                 (lptr_t)(sbase + (wave + i_ * F_NW) * 1024), 16, 0, 0);            \
            else                                                                                                    \
                __builtin_amdgcn_global_load_lds((gptr_t)(w_k + (t_).off[i_]),                                      \
                                                 (lptr_t)(sbase + F_BM * F_ROW_BYTES + (wave + (i_ - F_A_LOADS) * F_NW) * 1024), 16, 0, 0); \
        }                                                                                                           \
    } while (0)
    // (stage base, fragment offset, block offset): the two 16-byte halves of a lane's fragment
#define MT_F_READ(dst_, sb_, off_, blk_)                                                                            \
    do {                                                                                                            \
        const i32x4 lo_ = *reinterpret_cast<const i32x4*>((sb_) + (off_) + (blk_));                                 \
        const i32x4 hi_ = *reinterpret_cast<const i32x4*>((sb_) + ((off_) ^ 16) + (blk_));                          \
        dst_ = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);                                           \
    } while (0)
#define MT_F_MFMA(i_, j_) \
    acc[i_][j_] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[j_], af[i_], acc[i_][j_], 0, 0, 0, 0, 0, 0)

    i32x8 af[F_TMI], wf[F_TNI], wn[F_TNI];
    f32x16 acc[F_TMI][F_TNI];

    // ---- fill: slices 0 .. STAGES-1 of the first tile in flight; slice 0 landed for everyone and in registers
#pragma unroll
    for (int p = 0; p < STAGES; ++p) MT_F_ISSUE(cur, p, p);
    f_wait_vmcnt<F_LPS*(STAGES - 1)>();
    __builtin_amdgcn_s_barrier();
    {
        const unsigned char* sb = lds;
#pragma unroll
        for (int i = 0; i < F_TMI; ++i) MT_F_READ(af[i], sb, fa_off, i * 32 * F_ROW_BYTES);
#pragma unroll
        for (int j = 0; j < F_TNI; ++j) MT_F_READ(wf[j], sb, fw_off, j * 32 * F_ROW_BYTES);
    }
    int cs = 0;                                         // ring stage of slice kt (already in registers)

    constexpr int ROWB = F_PARK_ROWB, NCH = ROWB / 16, ROWS_PER_INST = 64 / NCH, NIT = 32 / ROWS_PER_INST;
    unsigned char* park = lds + RING_BYTES + wave * F_PARK_BYTES;
    const int c = lane % NCH;

    for (int j = 0; j < n_mine; ++j) {
        if (j + 1 < n_mine) locate(j + 1, nxt);
        else nxt = cur;                                 // no next tile: repeat loads of this one, never read
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);    // this lane's 4 bias values of the tile, fetched ahead of the epilogue
        {
            const float* __restrict__ bias = g.bias[cur.grp];
            const int nb = cur.n0 + wn0 + c * 4;
            if (bias && nb < s.N) bv = *reinterpret_cast<const float4*>(bias + nb);
        }
#pragma unroll
        for (int i = 0; i < F_TMI; ++i)
#pragma unroll
            for (int jj = 0; jj < F_TNI; ++jj)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

        // One K slice.  Sync point: this wavefront holds slice kt in registers (its reads are complete) and its own
        // loads of slice kt+1 have landed; after the barrier that holds for everyone, so the stage of slice kt takes
        // slice kt+STAGES (tile T_, slice R_) and slice kt+1 may be read.  No branch inside.
#define MT_F_SLICE(T_, R_)                                                                                          \
        do {                                                                                                        \
            const int ns = cs + 1 == STAGES ? 0 : cs + 1;                                                           \
            f_wait_lgkmcnt0();                                                                                      \
            f_wait_vmcnt<F_LPS*(STAGES - 2)>();                                                                     \
            __builtin_amdgcn_s_barrier();                                                                           \
            MT_F_ISSUE(T_, R_, cs);                                                                                 \
            const unsigned char* sb = lds + ns * F_STAGE_BYTES;                                                     \
            _Pragma("unroll") for (int jj = 0; jj < F_TNI; ++jj) MT_F_READ(wn[jj], sb, fw_off, jj * 32 * F_ROW_BYTES); \
            _Pragma("unroll") for (int i = 0; i < F_TMI; ++i) {                                                     \
                _Pragma("unroll") for (int jj = 0; jj < F_TNI; ++jj) MT_F_MFMA(i, jj);                              \
                MT_F_READ(af[i], sb, fa_off, i * 32 * F_ROW_BYTES);                                                 \
            }                                                                                                       \
            _Pragma("unroll") for (int jj = 0; jj < F_TNI; ++jj) wf[jj] = wn[jj];                                   \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            cs = ns;                                                                                                \
        } while (0)
        int kt = 0;
        for (; kt < KT - STAGES; ++kt) MT_F_SLICE(cur, kt + STAGES);
        for (kt = 0; kt < STAGES; ++kt) MT_F_SLICE(nxt, kt);
#undef MT_F_SLICE

        // ---- epilogue of tile `cur`, wavefront-private (see gemm_bf16_persist.hip): park a 32-row block, read all of it
        //      back, then scale / bias / activation / residual; output and residual through buffer instructions whose
        //      bounds check drops rows at or beyond M and lanes whose columns are beyond N
        {
            const float* __restrict__ res = g.residual[cur.grp];
            const float scale = g.scale[cur.grp];
            constexpr int ESZ = OUT == 1 ? 4 : (OUT == 0 ? 2 : 1);
            const uint32_t ldc_b = (uint32_t)s.ldc * ESZ, ldr_b = (uint32_t)s.ldr * 4;
            const __amdgpu_buffer_rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(g.C[cur.grp], 0, (int)((uint32_t)M * ldc_b), 0x00020000);
            const __amdgpu_buffer_rsrc_t r_rs =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(res ? res : (const float*)g.C[cur.grp]), 0, res ? (int)((uint32_t)M * ldr_b) : 0, 0x00020000);
            const int n = cur.n0 + wn0 + c * 4;
            const bool n_ok = n < s.N;                               // N % 4 == 0
            const uint32_t row0 = (uint32_t)(cur.m0 + wm0 + lane / NCH);
            const uint32_t c_off0 = n_ok ? row0 * ldc_b + (uint32_t)n * ESZ : 0x80000000u;
            const uint32_t r_off0 = n_ok ? row0 * ldr_b + (uint32_t)n * 4 : 0x80000000u;
            const float os = s.out_scale;
#pragma unroll
            for (int p = 0; p < F_TMI; ++p) {
                constexpr int GRP = OUT == 1 ? NIT / 2 : NIT;
                f32x4 rv[GRP];
                auto fetch_residual = [&](int it0) {
                    if constexpr (OUT == 1) {
                        if (res) {
#pragma unroll
                            for (int u = 0; u < GRP; ++u)
                                rv[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                                      r_rs, (int)(r_off0 + (uint32_t)(p * 32 + (it0 + u) * ROWS_PER_INST) * ldr_b), 0, 0));
                        }
                    }
                };
                fetch_residual(0);
                const int key_w = l32 & (NCH - 1);
#pragma unroll
                for (int jj = 0; jj < F_TNI; ++jj)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const int chunk = (jj * 32 + qq * 8 + half * 4) >> 2;
                        const f32x16& a = acc[p][jj];
                        *reinterpret_cast<float4*>(park + l32 * ROWB + ((chunk ^ key_w) << 4)) =
                            make_float4(a[qq * 4 + 0], a[qq * 4 + 1], a[qq * 4 + 2], a[qq * 4 + 3]);
                    }
#pragma unroll
                for (int it0 = 0; it0 < NIT; it0 += GRP) {
                    float4 v[GRP];
#pragma unroll
                    for (int u = 0; u < GRP; ++u) {
                        const int ml = (it0 + u) * ROWS_PER_INST + lane / NCH;
                        const int key = ml & (NCH - 1);
                        v[u] = *reinterpret_cast<const float4*>(park + ml * ROWB + ((c ^ key) << 4));
                    }
#pragma unroll
                    for (int u = 0; u < GRP; ++u) {
                        float4 o;
                        o.x = f_act<ACT>(fmaf(v[u].x, scale, bv.x));
                        o.y = f_act<ACT>(fmaf(v[u].y, scale, bv.y));
                        o.z = f_act<ACT>(fmaf(v[u].z, scale, bv.z));
                        o.w = f_act<ACT>(fmaf(v[u].w, scale, bv.w));
                        const int off = (int)(c_off0 + (uint32_t)(p * 32 + (it0 + u) * ROWS_PER_INST) * ldc_b);
                        if constexpr (OUT == 1) {
                            if (res) { o.x += rv[u][0]; o.y += rv[u][1]; o.z += rv[u][2]; o.w += rv[u][3]; }
                            const f32x4 ov = {o.x, o.y, o.z, o.w};
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, ov), c_rs, off, 0, 0);
                        } else if constexpr (OUT == 0) {
                            const bf16x4 ob = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
                            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, ob), c_rs, off, 0, 0);
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b32(pack_e4m3(o.x * os, o.y * os, o.z * os, o.w * os), c_rs, off, 0, 0);
                        }
                    }
                    if (it0 + GRP < NIT) fetch_residual(it0 + GRP);
                }
            }
        }
        cur = nxt;
    }
    f_wait_vmcnt<0>();                                   // repeat loads issued past the last tile must land before the LDS is released
#undef MT_F_ISSUE
#undef MT_F_READ
#undef MT_F_MFMA
}

template <int STAGES, int OUT, int ACT>
hipError_t f_launch_one(const GemmGroup& g, const GemmShape& s, int n_wg, hipStream_t stream)
{
    constexpr int LDS_BYTES = STAGES * F_STAGE_BYTES + F_NW * F_PARK_BYTES;
    const int tiles_n = (s.N + F_BN - 1) / F_BN;
    auto kfn = gemm_fp8_kernel<STAGES, OUT, ACT>;
    static std::atomic<uint64_t> lds_raised{0};
    hipError_t e = ensure_dynamic_lds((const void*)kfn, LDS_BYTES, lds_raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kfn, dim3(n_wg), dim3(F_NW * 64), LDS_BYTES, stream, g, s, tiles_n);
    return hipGetLastError();
}

int f_cu_count()
{
    static std::atomic<int> cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
    cached[dev].store(v, std::memory_order_relaxed);
    return v;
}

}  // namespace

hipError_t launch_gemm_fp8(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (s.G <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
    constexpr int ST = 3;
    // K slices of 64 must outnumber the ring stages (refills reach at most into the NEXT tile); 32-bit byte offsets
    if (s.G > kMaxGroup || s.splits != 1 || s.n_sub > 1 || s.d_sub_rows || s.K % 64 != 0 || s.K / 64 < ST || s.N % 4 != 0 || s.lda % 16 != 0 ||
        s.ldw % 16 != 0 || (s.ldw && s.ldw < s.K) || s.ldc % 4 != 0 || s.ldr % 4 != 0)
        return hipErrorInvalidValue;
    if ((uint64_t)s.M * (uint64_t)s.lda >= (1ull << 32) || (uint64_t)s.N * (uint64_t)(s.ldw ? s.ldw : s.K) >= (1ull << 32))
        return hipErrorInvalidValue;
    if (s.out_f32 != 1 && g.residual[0]) return hipErrorInvalidValue;
    // (output and residual are addressed through 32-bit buffer offsets with 0x80000000 as the "nowhere" offset)
    if ((uint64_t)s.M * (uint64_t)s.ldc * 4 >= (1ull << 31) || (uint64_t)s.M * (uint64_t)s.ldr * 4 >= (1ull << 31)) return hipErrorInvalidValue;
    const long tiles = (long)s.G * ((s.M + F_BM - 1) / F_BM) * ((s.N + F_BN - 1) / F_BN);
    const int n_wg = (int)std::min<long>(tiles, f_cu_count());
    const bool gelu = s.act == ACT_GELU_ERF || s.act == ACT_GELU_TANH;
    if (s.act != ACT_NONE && !gelu) return hipErrorInvalidValue;
    switch (s.out_f32) {
        case 1:
            if (s.act != ACT_NONE) return hipErrorInvalidValue;
            return f_launch_one<ST, 1, ACT_NONE>(g, s, n_wg, stream);
        case 0:
            if (s.act == ACT_GELU_ERF) return f_launch_one<ST, 0, ACT_GELU_ERF>(g, s, n_wg, stream);
            if (s.act == ACT_GELU_TANH) return f_launch_one<ST, 0, ACT_GELU_TANH>(g, s, n_wg, stream);
            return f_launch_one<ST, 0, ACT_NONE>(g, s, n_wg, stream);
        case 2:
            if (s.act == ACT_GELU_ERF) return f_launch_one<ST, 2, ACT_GELU_ERF>(g, s, n_wg, stream);
            if (s.act == ACT_GELU_TANH) return f_launch_one<ST, 2, ACT_GELU_TANH>(g, s, n_wg, stream);
            return f_launch_one<ST, 2, ACT_NONE>(g, s, n_wg, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace mt
