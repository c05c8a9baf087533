// bfloat16 contraction on the gfx950 matrix cores:
//   C_g[M,N] = epi(A_g[M,K] * W_g[N,K]^T),  g = 0..G-1 in ONE launch (one problem per active task).
// Both operands are K-contiguous, which is the native MFMA operand order, so no transposition is
// needed anywhere.  Accumulation is float32 (v_mfma_f32_32x32x16_bf16).
//
// Tiling.  A BM x BN output tile per workgroup, K consumed in slices of BK (32 or 64) elements
// through a ring of STAGES LDS stages.  Slices are fetched with global_load_lds_dwordx4: every lane
// moves 16 bytes from global memory straight into LDS, no staging registers and no LDS stores.  One
// such wavefront instruction fills 1024 contiguous LDS bytes (8 rows of 128 B or 16 rows of 64 B),
// lane l landing in 16-byte slot l of that span; a lane therefore FETCHES the chunk that belongs in
// its slot under the swizzle  slot = chunk ^ key(row), key = (row / rows-per-256-bytes) mod
// chunks-per-row, which spreads the 16-byte fragment reads of 16 consecutive rows over all banks.
//
// Pipeline.  One barrier per slice, placed at the start of the slice's last 16-wide K step, when all
// of a wavefront's fragment reads of that slice are in registers: after it the stage is free and is
// refilled with the slice STAGES ahead, the refill instructions being spread over the following K
// steps between MFMAs.  Fragments are double-buffered in registers so LDS latency hides behind the
// MFMAs of the previous step.
//
// Operand roles.  The weight fragment is the first MFMA operand and the activation fragment the
// second, so a lane ends up with 4 consecutive output columns n of one output row m: bias loads,
// residual loads and stores are 8- or 16-byte vectors along the row-major output.
//
// Workgroup -> tile mapping.  Consecutive workgroup ids go to different XCDs (8, each with its own
// L2), so ids are regrouped such that each XCD owns a contiguous range of tiles, and within a
// problem tiles are walked in bands of row-tiles so that concurrently resident tiles share weight
// columns and activation rows in that XCD's L2.
#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

#ifndef MT_GEMM_XCDS
#define MT_GEMM_XCDS 8
#endif
#ifndef MT_GEMM_BAND
#define MT_GEMM_BAND 8
#endif
#ifndef MT_GEMM_INTERLEAVE
#define MT_GEMM_INTERLEAVE 1
#endif
#ifndef MT_GEMM_BIG_TILE
#define MT_GEMM_BIG_TILE 9
#endif
#ifndef MT_GEMM_GELU_TILE
#define MT_GEMM_GELU_TILE 11
#endif
#ifndef MT_GEMM_WIDE_TILE
#define MT_GEMM_WIDE_TILE 19
#endif
#ifndef MT_GEMM_NARROW_TILE
#define MT_GEMM_NARROW_TILE 25
#endif
#ifndef MT_GEMM_DSPER
#define MT_GEMM_DSPER 1
#endif
constexpr int kXcds = MT_GEMM_XCDS;              // 1 disables the per-XCD regrouping of workgroup ids
constexpr bool kInterleave = MT_GEMM_INTERLEAVE != 0;
constexpr int kBand = MT_GEMM_BAND;              // row-tiles per raster band

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES>
struct GemmCfg {
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int CH = BK / 8;                       // 16-byte chunks per row
    static constexpr int KK = BK / 16;                      // MFMA K steps per slice
    static constexpr int RPI = 1024 / ROW_BYTES;            // rows filled by one wavefront load instruction
    static constexpr int KEY_SHIFT = (BK == 64) ? 1 : 2;    // rows per 256 bytes of LDS = 2 or 4
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TMI = WM / 32, TNI = WN / 32;
    static constexpr int A_LOADS = BM / RPI / NW, W_LOADS = BN / RPI / NW;   // load instructions per wavefront per slice
    static constexpr int LPS = A_LOADS + W_LOADS;
    static constexpr int LPP = (LPS + KK - 1) / KK;         // load instructions per K step ("part"), last part may be short
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(BM % (WAVES_M * 32) == 0 && BN % (WAVES_N * 32) == 0, "wave tile must be a multiple of 32x32");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "rows must split evenly over wavefront loads");
    static_assert(STAGES >= 2 && STAGES <= 8, "STAGES");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
    static_assert(LPS * (STAGES - 2) <= 63, "steady-state loads in flight exceed the 6-bit vmcnt");
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// wait until at most y*LPS of this wavefront's loads are outstanding (y = slices allowed in flight)
template <int LPS>
__device__ __forceinline__ void wait_slices(int y)
{
    constexpr int YMAX = (63 / LPS) < 6 ? (63 / LPS) : 6;     // vmcnt is a 6-bit counter
    if (y > YMAX) y = YMAX;
    if constexpr (YMAX >= 6) if (y == 6) { wait_vmcnt<6 * LPS>(); return; }
    if constexpr (YMAX >= 5) if (y == 5) { wait_vmcnt<5 * LPS>(); return; }
    if constexpr (YMAX >= 4) if (y == 4) { wait_vmcnt<4 * LPS>(); return; }
    if constexpr (YMAX >= 3) if (y == 3) { wait_vmcnt<3 * LPS>(); return; }
    if constexpr (YMAX >= 2) if (y == 2) { wait_vmcnt<2 * LPS>(); return; }
    if (y == 1) { wait_vmcnt<LPS>(); return; }
    wait_vmcnt<0>();
}

template <int ACT>
__device__ __forceinline__ float epi_act(float v)
{
    if constexpr (ACT == ACT_GELU_ERF) return gelu_erf_fast(v);
    else if constexpr (ACT == ACT_GELU_TANH) return gelu_tanh(v);
    else if constexpr (ACT == ACT_TANH) return tanhf(v);
    else return v;
}

// Interleave hint for one K step: NF fragment reads and NL global->LDS loads are slotted between the
// step's NM MFMAs so that no long run of non-MFMA instructions stalls the matrix pipe.
template <int LEFT, int P>
__device__ __forceinline__ void interleave_reads()
{
    if constexpr (LEFT > 0) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA ...
        __builtin_amdgcn_sched_group_barrier(0x100, LEFT < P ? LEFT : P, 0);     // ... then up to P fragment reads
        interleave_reads<(LEFT > P ? LEFT - P : 0), P>();
    }
}

template <int NM, int NF, int NL>
__device__ __forceinline__ void interleave_step()
{
    constexpr int P = MT_GEMM_DSPER;                       // fragment reads slotted behind each of the first MFMAs
    constexpr int a0 = (NF + P - 1) / P;
    constexpr int a = a0 < NM ? a0 : NM;
    constexpr int b = (NL < NM - a) ? NL : (NM - a);
    interleave_reads<NF, P>();
#pragma unroll
    for (int i = 0; i < b; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    if constexpr (NL > b) __builtin_amdgcn_sched_group_barrier(0x020, NL - b, 0);
    if constexpr (NM - a - b > 0) __builtin_amdgcn_sched_group_barrier(0x008, NM - a - b, 0);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int MINW, bool OUT_F32, int ACT, int FS>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, MINW) void gemm_bf16_kernel(GemmGroup g, GemmShape s, int tiles_n)
{
    using Cfg = GemmCfg<BM, BN, WAVES_M, WAVES_N, BK, STAGES>;
    constexpr int TMI = Cfg::TMI, TNI = Cfg::TNI, KK = Cfg::KK, ROW_BYTES = Cfg::ROW_BYTES, LPS = Cfg::LPS, LPP = Cfg::LPP;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // ---- rows actually present (the grid is sized for the bound s.M), then
    //      workgroup id -> (problem, row-tile, col-tile); workgroups beyond the last tile leave at once
    const int M = s.d_M ? min(s.M, *s.d_M) : s.M;
    const int tiles_m = (M + BM - 1) / BM;
    const int total = s.G * s.splits * tiles_m * tiles_n;
    if ((int)blockIdx.x >= total) return;
    int tile;
    {
        const int bid = blockIdx.x;
        const int x = bid % kXcds, i = bid / kXcds;
        const int q = total / kXcds, r = total % kXcds;
        tile = x * q + (x < r ? x : r) + i;
    }
    const int per_problem = tiles_m * tiles_n;
    const int gs = tile / per_problem;            // (problem, K range) pair; consecutive K ranges of a problem stay on one XCD
    const int grp = gs / s.splits, split = gs - grp * s.splits;
    const int t = tile - gs * per_problem;
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

    const int KT = s.K / BK / s.splits;           // slices of this workgroup's K range
    const unsigned char* __restrict__ A = static_cast<const unsigned char*>(g.A[grp]) + (size_t)split * KT * (BK * 2);
    const unsigned char* __restrict__ W = static_cast<const unsigned char*>(g.W[grp]) + (size_t)split * KT * (BK * 2);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / WAVES_N) * Cfg::WM, wn0 = (wave % WAVES_N) * Cfg::WN;
    const int l32 = lane & 31, half = lane >> 5;

    // ---- per-lane byte offsets of the 16-byte chunks this lane fetches (one per load instruction)
    // load i of a wavefront covers tile rows (wave + i*NW)*RPI .. +RPI-1; A loads first, then W loads
    uint32_t ld_off[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        const bool isA = i < Cfg::A_LOADS;
        const int row = (wave + (isA ? i : i - Cfg::A_LOADS) * Cfg::NW) * Cfg::RPI + lane / Cfg::CH;
        const int chunk = (lane % Cfg::CH) ^ ((row >> Cfg::KEY_SHIFT) & (Cfg::CH - 1));
        if (isA) ld_off[i] = (uint32_t)min(m0 + row, M - 1) * (uint32_t)(s.lda * 2) + chunk * 16;
        else ld_off[i] = (uint32_t)min(n0 + row, s.N - 1) * (uint32_t)((s.ldw ? s.ldw : s.K) * 2) + chunk * 16;
    }

    f32x16 acc[TMI][TNI];
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fragment read offsets inside a stage: row r = l32 of a 32-row block, K step kk -> slot (2kk+half) ^ key(r)
    int fa_off[KK], fw_off[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int o = l32 * ROW_BYTES + (((kk * 2 + half) ^ ((l32 >> Cfg::KEY_SHIFT) & (Cfg::CH - 1))) << 4);
        fa_off[kk] = wm0 * ROW_BYTES + o;
        fw_off[kk] = (BM + wn0) * ROW_BYTES + o;
    }


    // issue load instructions [part*LPP, part*LPP+LPP) of slice kt_ (caller guarantees kt_ < KT)
#define MT_ISSUE_PART(kt_, part_)                                                                                  \
    do {                                                                                                           \
        const unsigned char* a_k = A + (size_t)(kt_) * ROW_BYTES;                                                  \
        const unsigned char* w_k = W + (size_t)(kt_) * ROW_BYTES;                                                  \
        unsigned char* sbase = lds + ((kt_) % STAGES) * Cfg::STAGE_BYTES;                                          \
        _Pragma("unroll") for (int i_ = (part_) * LPP; i_ < (part_) * LPP + LPP; ++i_) {                           \
            if (i_ >= LPS) {} else if (i_ < Cfg::A_LOADS)                                                                               \
                __builtin_amdgcn_global_load_lds((gptr_t)(a_k + ld_off[i_]),                                       \
                                                 (lptr_t)(sbase + (wave + i_ * Cfg::NW) * 1024), 16, 0, 0);        \
            else                                                                                                   \
                __builtin_amdgcn_global_load_lds((gptr_t)(w_k + ld_off[i_]),                                       \
                                                 (lptr_t)(sbase + BM * ROW_BYTES + (wave + (i_ - Cfg::A_LOADS) * Cfg::NW) * 1024), 16, 0, 0); \
        }                                                                                                          \
    } while (0)

#define MT_LOAD_FRAGS(buf_, kt_, kk_)                                                                              \
    do {                                                                                                           \
        const unsigned char* sb = lds + ((kt_) % STAGES) * Cfg::STAGE_BYTES;                                       \
        _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                            \
            af[buf_][i] = *reinterpret_cast<const bf16x8*>(sb + fa_off[kk_] + i * 32 * ROW_BYTES);                 \
        _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                            \
            wf[buf_][j] = *reinterpret_cast<const bf16x8*>(sb + fw_off[kk_] + j * 32 * ROW_BYTES);                 \
    } while (0)

#define MT_MFMAS(buf_)                                                                                             \
    do {                                                                                                           \
        _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                            \
            _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                        \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf_][j], af[buf_][i], acc[i][j], 0, 0, 0); \
    } while (0)

    if constexpr (FS) {
        // ---- slice-scope fragment buffers: ALL fragments of slice kt+1 are read while the MFMAs of slice kt
        // run, so the LDS read latency hides behind a whole slice of MFMAs (tiles with few MFMAs per K step
        // cannot hide it behind one step).  Per slice: wait own reads of slice kt and own loads of slice
        // kt+1, barrier (stage kt is free, slice kt+1 is complete), refill stage kt, read slice kt+1,
        // multiply slice kt.
        bf16x8 afs[2][KK][TMI], wfs[2][KK][TNI];
#define MT_LOAD_SLICE(buf_, kt_)                                                                                   \
    do {                                                                                                           \
        const unsigned char* sb = lds + ((kt_) % STAGES) * Cfg::STAGE_BYTES;                                       \
        _Pragma("unroll") for (int kk = 0; kk < KK; ++kk) {                                                        \
            _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                        \
                afs[buf_][kk][i] = *reinterpret_cast<const bf16x8*>(sb + fa_off[kk] + i * 32 * ROW_BYTES);         \
            _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                        \
                wfs[buf_][kk][j] = *reinterpret_cast<const bf16x8*>(sb + fw_off[kk] + j * 32 * ROW_BYTES);         \
        }                                                                                                          \
    } while (0)
#define MT_MFMA_SLICE(buf_)                                                                                        \
    do {                                                                                                           \
        _Pragma("unroll") for (int kk = 0; kk < KK; ++kk)                                                          \
            _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                        \
                _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                    \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfs[buf_][kk][j], afs[buf_][kk][i], acc[i][j], 0, 0, 0); \
    } while (0)
#define MT_ISSUE_SLICE(kt_)                                                                                        \
    do {                                                                                                           \
        _Pragma("unroll") for (int part = 0; part < KK; ++part) MT_ISSUE_PART(kt_, part);                          \
    } while (0)
        // one slice in the steady state (its refill exists): buffer index is a compile-time constant
#define MT_STEADY(kt_, buf_)                                                                                       \
    do {                                                                                                           \
        wait_lgkmcnt0();                                                                                           \
        wait_vmcnt<LPS*(STAGES - 2)>();                                                                            \
        __builtin_amdgcn_s_barrier();                                                                              \
        MT_ISSUE_SLICE((kt_) + STAGES);                                                                            \
        MT_LOAD_SLICE((buf_) ^ 1, (kt_) + 1);                                                                      \
        MT_MFMA_SLICE(buf_);                                                                                       \
        if constexpr (kInterleave) interleave_step<TMI * TNI * KK, (TMI + TNI) * KK, LPS>();                       \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
    } while (0)
        // one slice of the tail: the refill and even the next slice may not exist
#define MT_TAIL(kt_, buf_)                                                                                         \
    do {                                                                                                           \
        wait_lgkmcnt0();                                                                                           \
        if ((kt_) + 1 < KT) {                                                                                      \
            wait_slices<LPS>(min(KT - 2 - (kt_), STAGES - 2));                                                     \
            __builtin_amdgcn_s_barrier();                                                                          \
            if ((kt_) + STAGES < KT) MT_ISSUE_SLICE((kt_) + STAGES);                                               \
            MT_LOAD_SLICE((buf_) ^ 1, (kt_) + 1);                                                                  \
        }                                                                                                          \
        MT_MFMA_SLICE(buf_);                                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
    } while (0)

#pragma unroll
        for (int p = 0; p < STAGES - 1; ++p)
            if (p < KT) MT_ISSUE_SLICE(p);
        wait_slices<LPS>(min(STAGES - 2, KT - 1));
        __builtin_amdgcn_s_barrier();
        if (STAGES - 1 < KT) MT_ISSUE_SLICE(STAGES - 1);
        MT_LOAD_SLICE(0, 0);
        const int KT_pairs = (max(0, KT - STAGES) & ~1);      // slices handled two at a time, every refill exists
        int kt = 0;
        for (; kt < KT_pairs; kt += 2) {
            MT_STEADY(kt, 0);
            MT_STEADY(kt + 1, 1);
        }
        for (; kt < KT; kt += 2) {
            MT_TAIL(kt, 0);
            if (kt + 1 < KT) MT_TAIL(kt + 1, 1);
        }
#undef MT_LOAD_SLICE
#undef MT_MFMA_SLICE
#undef MT_ISSUE_SLICE
#undef MT_STEADY
#undef MT_TAIL
    } else {
    bf16x8 af[2][TMI], wf[2][TNI];
    
        // prologue: slices 0..STAGES-2 in flight, wait for slice 0, then start refilling like a sync point would
    #pragma unroll
        for (int p = 0; p < STAGES - 1; ++p)
            if (p < KT) {
    #pragma unroll
                for (int part = 0; part < KK; ++part) MT_ISSUE_PART(p, part);
            }
        wait_slices<LPS>(min(STAGES - 2, KT - 1));
        __builtin_amdgcn_s_barrier();
        if (STAGES - 1 < KT) MT_ISSUE_PART(STAGES - 1, 0);
        MT_LOAD_FRAGS(0, 0, 0);
    
        // steady state: every refill exists, no conditionals inside
        const int KT_main = max(0, KT - STAGES);
        int kt = 0;
        for (; kt < KT_main; ++kt) {
    #pragma unroll
            for (int kk = 0; kk < KK - 1; ++kk) {
                MT_LOAD_FRAGS((kk + 1) & 1, kt, kk + 1);
                MT_ISSUE_PART(kt + STAGES - 1, kk + 1);
                MT_MFMAS(kk & 1);
                if constexpr (kInterleave) interleave_step<TMI * TNI, TMI + TNI, LPP>();
                __builtin_amdgcn_sched_barrier(0);
            }
            // sync point: this wavefront's reads of slice kt are in registers; slice kt+1 must have landed
            wait_lgkmcnt0();
            wait_vmcnt<LPS*(STAGES - 2)>();
            __builtin_amdgcn_s_barrier();
            MT_ISSUE_PART(kt + STAGES, 0);          // stage kt % STAGES was just vacated by everyone
            MT_LOAD_FRAGS(0, kt + 1, 0);
            MT_MFMAS((KK - 1) & 1);
            if constexpr (kInterleave) interleave_step<TMI * TNI, TMI + TNI, LPP>();
            __builtin_amdgcn_sched_barrier(0);
        }
        // drain: the last min(KT, STAGES) slices; only slice KT-1 may still lack its parts 1..KK-1
        if (kt + STAGES - 1 < KT) {
    #pragma unroll
            for (int part = 1; part < KK; ++part) MT_ISSUE_PART(kt + STAGES - 1, part);
        }
        for (; kt < KT; ++kt) {
    #pragma unroll
            for (int kk = 0; kk < KK - 1; ++kk) {
                MT_LOAD_FRAGS((kk + 1) & 1, kt, kk + 1);
                MT_MFMAS(kk & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kt + 1 < KT) {
                wait_lgkmcnt0();
                wait_slices<LPS>(KT - 1 - (kt + 1));
                __builtin_amdgcn_s_barrier();
                MT_LOAD_FRAGS(0, kt + 1, 0);
            }
            MT_MFMAS((KK - 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef MT_ISSUE_PART
#undef MT_LOAD_FRAGS
#undef MT_MFMAS

    // ---- epilogue.  A lane holds, for block (i,j): row m = ..+l32, columns n = ..+8*q+4*half+{0..3}, q=0..3.
    // Storing that layout directly would touch 32 rows with 16 bytes each per instruction, and would
    // re-load the bias for every block.  Instead every wavefront parks its raw float32 accumulators
    // in its own slice of the now idle LDS ring and reads them back row-contiguously, 4 consecutive
    // columns per lane: the lane's 4 bias values are loaded once, bias / activation / residual are
    // applied in a short rolled loop, and the stores cover whole row segments.
    constexpr int ROWB = Cfg::WN * 4;                         // bytes per parked row
    constexpr int NCH = ROWB / 16;                            // 16-byte chunks per row = lanes per row on the way out
    constexpr int RPW = ROWB >= 256 ? 1 : 256 / ROWB;         // rows per 256 bytes: swizzle key = (row / RPW) mod NCH
    constexpr int REGION = (Cfg::LDS_BYTES / Cfg::NW) & ~1023;
    constexpr int RPP = (REGION / ROWB >= Cfg::WM) ? Cfg::WM : ((REGION / ROWB >= 64) ? 64 : 32);   // rows per pass
    static_assert(REGION / ROWB >= 32 && Cfg::WM % RPP == 0, "LDS ring too small to park a 32-row block");
    static_assert(NCH <= 64 && 64 % NCH == 0, "row must split evenly over lanes");
    constexpr int ROWS_PER_INST = 64 / NCH;
    unsigned char* park = lds + wave * REGION;
    const int c = lane % NCH;
    const int n = n0 + wn0 + c * 4;
    const bool n_ok = n < s.N;                                // N % 4 == 0, so the lane's 4 columns are all in or all out
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (g.bias[grp] && n_ok) bv = *reinterpret_cast<const float4*>(g.bias[grp] + n);
    const float* __restrict__ res = g.residual[grp];
    unsigned char* __restrict__ Cout = static_cast<unsigned char*>(g.C[grp]) + (size_t)split * s.split_stride * 4;   // hoisted
    const size_t ldc_b = (size_t)s.ldc * (OUT_F32 ? 4 : 2), ldr_b = (size_t)s.ldr * 4;
    constexpr int NIT = RPP / ROWS_PER_INST;                 // read-back iterations per pass
    constexpr int UNR = NIT >= 4 ? 4 : 1;                      // LDS reads in flight per lane
    // residual rows of a pass are fetched up front so that their HBM latency overlaps the parking:
    // as many as the register budget allows (the rest are fetched late, UNR at a time)
    constexpr int PF = !OUT_F32 ? 0 : (MINW >= 2 ? (NIT < 8 ? NIT : 8) : (NIT < 32 ? NIT : 32));

    __builtin_amdgcn_s_barrier();      // every wavefront has taken its last fragments out of the ring
#pragma unroll
    for (int p = 0; p < Cfg::WM / RPP; ++p) {
        float4 rpf[PF > 0 ? PF : 1];
        if constexpr (PF > 0) {
            if (res) {
                const int nc = n_ok ? n : 0;
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int mc = min(m0 + wm0 + p * RPP + u * ROWS_PER_INST + lane / NCH, M - 1);
                    rpf[u] = *reinterpret_cast<const float4*>(reinterpret_cast<const unsigned char*>(res) + mc * ldr_b + nc * 4);
                }
            }
        }
#pragma unroll
        for (int ii = 0; ii < RPP / 32; ++ii) {
            const int ml = ii * 32 + l32;
            const int key = (ml / RPW) & (NCH - 1);
#pragma unroll
            for (int j = 0; j < TNI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int chunk = (j * 32 + q * 8 + half * 4) >> 2;
                    const f32x16& a = acc[p * (RPP / 32) + ii][j];
                    *reinterpret_cast<float4*>(park + ml * ROWB + ((chunk ^ key) << 4)) =
                        make_float4(a[q * 4 + 0], a[q * 4 + 1], a[q * 4 + 2], a[q * 4 + 3]);
                }
        }
        // the same wavefront reads back what it wrote: LDS operations of one wavefront execute in order
#pragma unroll
        for (int it = 0; it < NIT; it += UNR) {
            float4 v[UNR], rv[UNR];
            int mm[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {                             // unconditional, in-bounds reads first
                const int ml = (it + u) * ROWS_PER_INST + lane / NCH;
                const int key = (ml / RPW) & (NCH - 1);
                v[u] = *reinterpret_cast<const float4*>(park + ml * ROWB + ((c ^ key) << 4));
                mm[u] = m0 + wm0 + p * RPP + ml;
                if constexpr (OUT_F32) {
                    if (res) {
                        if (it + u < PF) rv[u] = rpf[(it + u) < PF ? (it + u) : 0];
                        else {
                            const int mc = min(mm[u], M - 1);
                            const int nc = n_ok ? n : 0;
                            rv[u] = *reinterpret_cast<const float4*>(reinterpret_cast<const unsigned char*>(res) + mc * ldr_b + nc * 4);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                float4 o;
                o.x = epi_act<ACT>(v[u].x + bv.x);
                o.y = epi_act<ACT>(v[u].y + bv.y);
                o.z = epi_act<ACT>(v[u].z + bv.z);
                o.w = epi_act<ACT>(v[u].w + bv.w);
                const bool ok = n_ok && mm[u] < M;
                if constexpr (OUT_F32) {
                    if (res) { o.x += rv[u].x; o.y += rv[u].y; o.z += rv[u].z; o.w += rv[u].w; }
                    if (ok) *reinterpret_cast<float4*>(Cout + mm[u] * ldc_b + n * 4) = o;
                } else {
                    bf16x4 ob = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
                    if (ok) *reinterpret_cast<bf16x4*>(Cout + mm[u] * ldc_b + n * 2) = ob;
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int MINW, bool OUT_F32, int ACT, int FS>
hipError_t launch_one(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    using Cfg = GemmCfg<BM, BN, WAVES_M, WAVES_N, BK, STAGES>;
    const int tiles_m = (s.M + BM - 1) / BM, tiles_n = (s.N + BN - 1) / BN;
    const int total = s.G * s.splits * tiles_m * tiles_n;
    if (s.K % (BK * s.splits) != 0) return hipErrorInvalidValue;
    auto kfn = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, OUT_F32, ACT, FS>;
    static std::atomic<uint64_t> lds_raised{0};          // one per instantiation
    if (Cfg::LDS_BYTES > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kfn, Cfg::LDS_BYTES, lds_raised);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kfn, dim3(total), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, g, s, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int MINW, int FS = 0>
hipError_t launch_cfg(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    // Instantiated epilogues: float32 output without activation (residual sums feeding LayerNorm) or with
    // tanh (pooler), and bf16 output with none / GELU(erf) / GELU(tanh).
    if (s.out_f32) {
        if (s.act == ACT_TANH) return launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, true, ACT_TANH, FS>(g, s, stream);
        if (s.act != ACT_NONE) return hipErrorInvalidValue;
        return launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, true, ACT_NONE, FS>(g, s, stream);
    }
    switch (s.act) {
        case ACT_NONE: return launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, false, ACT_NONE, FS>(g, s, stream);
        case ACT_GELU_ERF: return launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, false, ACT_GELU_ERF, FS>(g, s, stream);
        case ACT_GELU_TANH: return launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, MINW, false, ACT_GELU_TANH, FS>(g, s, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

int g_gemm_bf16_tile_override = 0;   // 0 = choose by shape; set through mt_debug_set_gemm_tile for tuning sweeps

hipError_t launch_gemm_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (s.G <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
    if (s.splits < 1 || (s.splits > 1 && (!s.out_f32 || s.act != ACT_NONE || g.bias[0] || g.residual[0]))) return hipErrorInvalidValue;
    if (s.K % 64 != 0 || s.K < 64 || s.N % 4 != 0 || s.lda % 8 != 0 || s.ldw % 8 != 0 || (s.ldw && s.ldw < s.K) || s.ldc % 4 != 0 || s.ldr % 4 != 0 ||
        s.G > kMaxGroup || (!s.out_f32 && g.residual[0] != nullptr))
        return hipErrorInvalidValue;
    // per-lane chunk offsets are 32-bit
    if ((uint64_t)s.M * (uint64_t)s.lda * 2 >= (1ull << 32) || (uint64_t)s.N * (uint64_t)(s.ldw ? s.ldw : s.K) * 2 >= (1ull << 32))
        return hipErrorInvalidValue;
    int sel = g_gemm_bf16_tile_override;
    // workgroups a 64x128 tiling of the launch would have
    const long wg64 = (long)s.G * s.splits * ((s.M + 63) / 64) * ((s.N + 127) / 128);
    // Few rows: the weight-streaming kernel, unless the launch still fills a good part of the chip with tiles (several
    // problems with wide outputs, or 512 rows and more in all): measured at 64..256 rows, 1 and 8 problems, the tiled
    // kernel is then 1.3x to 3.5x faster.  K-split launches and launches of fewer than 64 rows (half-empty tiles) stay
    // with the streaming kernel.
    const bool few_rows = s.M <= 256 && !(s.splits == 1 && s.M >= 64 && (wg64 >= 64 || (long)s.G * s.M >= 512));
    if ((sel == 0 && few_rows) || sel == 13 || s.n_sub > 1 || s.d_sub_rows) {
        return launch_gemm_skinny_bf16(g, s, stream);
    }
    if (sel == 27) return launch_gemm_bf16_persist(g, s, stream);
    if (sel == 0 && gemm_bf16_persist_wants(s)) return launch_gemm_bf16_persist(g, s, stream);
    if (sel == 0) {
        // Shape rule from measurements on MI355X (BERT-base widths, 1 and 8 problems, 2304 and 4096 rows).
        // The row bound s.M over-counts when padding is dropped on the device, so the rule keys on the
        // number of 256x256 tiles the bound implies and errs towards the smaller tile when few.
        //   many tiles: 256x256 with 8 wavefronts (least L2 traffic per flop); the GELU epilogue's vector
        //   work instead prefers 8 wavefronts of 64x64 on a 256x128 tile, two workgroups per CU;
        //   few tiles (single problem): 128x128 (wide outputs) or 64x128 (narrow outputs, and wide ones of up to about
        //   1024 rows, where 128x128 tiles leave most CUs without work), two workgroups per CU,
        //   slice-scope fragment buffers (4 MFMAs per K step cannot hide an LDS read behind one step).
        const long t256 = (long)s.G * s.splits * ((s.M + 255) / 256) * ((s.N + 255) / 256);
        const bool gelu = s.act == ACT_GELU_ERF || s.act == ACT_GELU_TANH;
        // (a short, narrow product - the attention output projection - also prefers the 256x128 tile: 72 vs 80 us
        //  for 8 problems of 4096 x 768 x 768)
        if (t256 >= 256) sel = (gelu || (s.N <= 1024 && s.K <= 1024)) ? MT_GEMM_GELU_TILE : MT_GEMM_BIG_TILE;
        else if (s.N >= 2048 && wg64 > 400) sel = MT_GEMM_WIDE_TILE;
        else sel = MT_GEMM_NARROW_TILE;                      // narrow output: 64-row tiles double the tile count, so K needs less splitting
    }
    switch (sel) {
        case 2: return launch_cfg<256, 128, 2, 2, 32, 3, 2>(g, s, stream);   // 72 KB LDS: two workgroups per CU
        case 3: return launch_cfg<256, 256, 2, 2, 32, 4, 1>(g, s, stream);   // 128 KB LDS, 128x128 per wavefront
        case 4: return launch_cfg<256, 256, 2, 4, 64, 2, 2>(g, s, stream);   // 8 wavefronts
        case 5: return launch_cfg<128, 256, 2, 2, 32, 3, 2>(g, s, stream);
        case 6: return launch_cfg<128, 128, 2, 2, 64, 2, 2>(g, s, stream);   // 64 KB LDS: two workgroups per CU
        case 7: return launch_cfg<256, 256, 2, 2, 64, 2, 1>(g, s, stream);
        case 8: return launch_cfg<256, 128, 2, 2, 64, 3, 1>(g, s, stream);
        case 9: return launch_cfg<256, 256, 2, 4, 32, 4, 2>(g, s, stream);
        case 10: return launch_cfg<256, 128, 2, 2, 64, 2, 1>(g, s, stream);
        case 11: return launch_cfg<256, 128, 4, 2, 32, 3, 2>(g, s, stream);  // 8 wavefronts of 64x64, 72 KB
        case 12: return launch_cfg<128, 128, 2, 2, 32, 3, 2>(g, s, stream);  // 48 KB: three workgroups per CU
        case 14: return launch_cfg<128, 128, 2, 2, 64, 4, 1>(g, s, stream);  // 128 KB: 3 slices of 64 ahead
        case 15: return launch_cfg<128, 128, 2, 2, 32, 8, 1>(g, s, stream);  // 128 KB: 7 slices of 32 ahead
        case 16: return launch_cfg<256, 128, 4, 2, 32, 6, 1>(g, s, stream);  // 144 KB, 8 wavefronts
        case 17: return launch_cfg<128, 128, 2, 2, 32, 6, 1>(g, s, stream);  // 96 KB
        // slice-scope fragment buffers
        case 18: return launch_cfg<128, 128, 2, 2, 32, 3, 2, 1>(g, s, stream);
        case 19: return launch_cfg<128, 128, 2, 2, 64, 2, 2, 1>(g, s, stream);
        case 20: return launch_cfg<128, 128, 2, 2, 32, 4, 2, 1>(g, s, stream);
        case 21: return launch_cfg<256, 128, 4, 2, 32, 3, 2, 1>(g, s, stream);
        case 22: return launch_cfg<256, 256, 2, 4, 32, 4, 2, 1>(g, s, stream);
        case 23: return launch_cfg<128, 128, 2, 2, 32, 5, 2, 1>(g, s, stream);  // 80 KB: two workgroups per CU, 4 slices ahead
        case 24: return launch_cfg<64, 128, 2, 2, 32, 4, 2, 1>(g, s, stream);   // 48 KB: narrow outputs without a K split
        case 25: return launch_cfg<64, 128, 2, 2, 64, 3, 2, 1>(g, s, stream);   // 72 KB
        case 26: return launch_cfg<64, 256, 2, 2, 32, 4, 2, 1>(g, s, stream);   // 80 KB
        default: return launch_cfg<128, 128, 2, 2, 32, 4, 2>(g, s, stream);  // 64 KB LDS
    }
}

}  // namespace mt
