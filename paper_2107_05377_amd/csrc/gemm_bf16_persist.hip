// Persistent form of the bfloat16 contraction  C_g[M,N] = epi(A_g[M,K] * W_g[N,K]^T)  for launches with more
// output tiles than the chip has compute units.
//
// The one-tile-per-workgroup kernel pays, per tile, a pipeline fill (nothing to multiply until the first K slice
// has crossed the chip) and an epilogue during which its compute unit multiplies nothing; since all tiles of a
// round start together, all epilogues also hit memory together.  Here one workgroup per compute unit walks a
// list of tiles and never lets its load ring drain:
//   - the ring of STAGES K slices (global_load_lds: global memory straight into LDS, XOR-swizzled 16-byte
//     chunks, see gemm_bf16.hip) is indexed by a slice counter that runs across tiles: while the last slices of a
//     tile are multiplied, the first slices of the workgroup's NEXT tile are already being fetched, and the
//     first fragments of the next tile are in registers when the epilogue starts;
//   - the epilogue has an LDS region of its own (one 32-row block of the wavefront's sub-tile at a time, private
//     to the wavefront, so it needs no barrier), because the ring is busy with the next tile's slices;
//   - stores are issued and left behind; the wavefront goes straight on to the next tile's slices.
// Every wavefront executes the same number of barriers: all loops are uniform over the workgroup, and a
// workgroup without a next tile issues harmless repeat loads of its current tile so that the wait counts of the
// steady state hold for every slice.
//
// Tile 256 x 256, K slices of 32, 8 wavefronts of 128 x 64 (v_mfma_f32_32x32x16_bf16, float32 accumulation).
// Workgroup -> tile list: workgroup ids go round-robin over the 8 XCDs (each with its own L2); XCD x owns a
// contiguous range of the tile order, and its workgroups take that range in strides of the XCD's workgroup
// count, so the tiles an XCD works on at any time are neighbours (same activation rows or weight columns).
#include <algorithm>

#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int kPXcds = 8;
constexpr int kPBand = 8;              // row-tiles per raster band

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int N>
__device__ __forceinline__ void p_wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void p_wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int ACT>
__device__ __forceinline__ float p_act(float v)
{
    if constexpr (ACT == ACT_GELU_ERF) return gelu_erf_fast(v);
    else if constexpr (ACT == ACT_GELU_TANH) return gelu_tanh(v);
    else if constexpr (ACT == ACT_TANH) return tanhf(v);
    else return v;
}

// One K step's instruction mix for the scheduler: NM MFMAs; the NF fragment reads go behind the first MFMAs,
// PER at a time, so that the rest of the step's MFMAs cover their latency before the next step needs them; the NL
// global->LDS loads follow, one per MFMA.
template <int NM, int NF, int NL, int PER>
__device__ __forceinline__ void p_interleave()
{
    if constexpr (NM > 0) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   // one MFMA ...
        if constexpr (NF > 0) {
            __builtin_amdgcn_sched_group_barrier(0x100, NF < PER ? NF : PER, 0);              // ... then fragment reads
            p_interleave<NM - 1, (NF > PER ? NF - PER : 0), NL, PER>();
        } else if constexpr (NL > 0) {
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                               // ... or one load
            p_interleave<NM - 1, 0, NL - 1, PER>();
        } else {
            p_interleave<NM - 1, 0, 0, PER>();
        }
    }
}

#ifndef MT_P_DSPER
#define MT_P_DSPER 2
#endif

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK_, int STAGES, int PARK_COLS_>
struct PCfg {
    static constexpr int BK = BK_, ROW_BYTES = BK * 2, CH = BK / 8, KK = BK / 16, RPI = 1024 / ROW_BYTES;
    static constexpr int KEY_SHIFT = (BK == 64) ? 1 : 2;     // rows per 256 bytes of LDS = 2 or 4
    static constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TMI = WM / 32, TNI = WN / 32;
    static constexpr int A_LOADS = BM / RPI / NW, W_LOADS = BN / RPI / NW, LPS = A_LOADS + W_LOADS;
    static constexpr int LPP = LPS / KK;
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int RING_BYTES = STAGES * STAGE_BYTES;
    static constexpr int PARK_COLS = PARK_COLS_;             // columns of the wavefront's sub-tile parked at a time (WN or 32)
    static constexpr int PARK_ROWB = PARK_COLS * 4;          // bytes per parked float32 row
    static constexpr int PARK_BYTES = 32 * PARK_ROWB;        // one 32-row block
    static constexpr int LDS_BYTES = RING_BYTES + NW * PARK_BYTES;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "rows must split evenly over wavefront loads");
    static_assert(LPS % KK == 0, "loads of a slice must split evenly over its K steps");
    static_assert(STAGES >= 2 && LPS * (STAGES - 2) <= 63, "ring depth");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(PARK_COLS == WN || PARK_COLS == 32, "park block");
};

// What a workgroup needs to know of one tile to fetch it.
template <int LPS>
struct TileRef {
    const unsigned char* A;
    const unsigned char* W;
    uint32_t off[LPS];     // per load instruction: this lane's byte offset of its 16-byte chunk (row * stride + swizzled chunk)
    int grp, m0, n0;
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int PARK_COLS, bool OUT_F32, int ACT>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, 1) void gemm_bf16_persist_kernel(GemmGroup g, GemmShape s, int tiles_n, int band_rows)
{
    using Cfg = PCfg<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS>;
    constexpr int KK = Cfg::KK;
    constexpr int TMI = Cfg::TMI, TNI = Cfg::TNI, ROW_BYTES = Cfg::ROW_BYTES, LPS = Cfg::LPS, LPP = Cfg::LPP;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int M = s.d_M ? min(s.M, *s.d_M) : s.M;
    const int tiles_m = (M + BM - 1) / BM;
    const int per_problem = tiles_m * tiles_n;
    const int total = s.G * per_problem;
    // this workgroup's tiles: XCD x owns tiles [lo, lo + cnt), its workgroups stride through them
    const int xcd = blockIdx.x % kPXcds, wi = blockIdx.x / kPXcds;
    const int wg_x = ((int)gridDim.x - xcd + kPXcds - 1) / kPXcds;          // workgroups of this launch on XCD x
    const int q = total / kPXcds, r = total % kPXcds;
    const int lo = xcd * q + min(xcd, r), cnt = q + (xcd < r ? 1 : 0);
    if (wi >= cnt) return;                                                   // uniform over the workgroup
    const int n_mine = (cnt - wi + wg_x - 1) / wg_x;

    const int KT = s.K / BK;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / WAVES_N) * Cfg::WM, wn0 = (wave % WAVES_N) * Cfg::WN;
    const int l32 = lane & 31, half = lane >> 5;
    const uint32_t lda_b = (uint32_t)(s.lda * 2), ldw_b = (uint32_t)((s.ldw ? s.ldw : s.K) * 2);

    // rows of the tile covered by this lane's load instructions, and the chunk it fetches (the swizzle puts chunk
    // c of row r into slot c ^ key(r), so the lane that FILLS slot l % CH fetches chunk (l % CH) ^ key(r))
    int ld_row[LPS], ld_chunk[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        const bool isA = i < Cfg::A_LOADS;
        ld_row[i] = (wave + (isA ? i : i - Cfg::A_LOADS) * Cfg::NW) * Cfg::RPI + lane / Cfg::CH;
        ld_chunk[i] = ((lane % Cfg::CH) ^ ((ld_row[i] >> Cfg::KEY_SHIFT) & (Cfg::CH - 1))) * 16;
    }
    auto locate = [&](int j, TileRef<LPS>& t) {      // j-th tile of this workgroup
        const int tile = lo + wi + j * wg_x;
        t.grp = tile / per_problem;
        const int tt = tile - t.grp * per_problem;
        const int band_sz = band_rows * tiles_n;
        const int band = tt / band_sz;
        const int rows_in_band = min(band_rows, tiles_m - band * band_rows);
        const int tb = tt - band * band_sz;
        const int tn = tb / rows_in_band;
        const int tm = band * band_rows + tb % rows_in_band;
        t.m0 = tm * BM;
        t.n0 = tn * BN;
        t.A = static_cast<const unsigned char*>(g.A[t.grp]);
        t.W = static_cast<const unsigned char*>(g.W[t.grp]);
#pragma unroll
        for (int i = 0; i < LPS; ++i) {
            if (i < Cfg::A_LOADS) t.off[i] = (uint32_t)min(t.m0 + ld_row[i], M - 1) * lda_b + ld_chunk[i];
            else t.off[i] = (uint32_t)min(t.n0 + ld_row[i], s.N - 1) * ldw_b + ld_chunk[i];
        }
    };

    // fragment read offsets inside a stage: row l32 of a 32-row block, K step kk -> slot (2kk + half) ^ key(row)
    int fa_off[Cfg::KK], fw_off[Cfg::KK];
#pragma unroll
    for (int kk = 0; kk < Cfg::KK; ++kk) {
        const int o = l32 * ROW_BYTES + (((kk * 2 + half) ^ ((l32 >> Cfg::KEY_SHIFT) & (Cfg::CH - 1))) << 4);
        fa_off[kk] = wm0 * ROW_BYTES + o;
        fw_off[kk] = (BM + wn0) * ROW_BYTES + o;
    }

    TileRef<LPS> cur, nxt;
    locate(0, cur);

    // load instructions [part*LPP, part*LPP+LPP) of K slice `slice_` of tile `t_` into ring stage `stage_`
#define MT_P_ISSUE(t_, slice_, stage_, part_)                                                                       \
    do {                                                                                                            \
        const unsigned char* a_k = (t_).A + (size_t)(slice_) * ROW_BYTES;                                           \
        const unsigned char* w_k = (t_).W + (size_t)(slice_) * ROW_BYTES;                                           \
        unsigned char* sbase = lds + (stage_) * Cfg::STAGE_BYTES;                                                   \
        _Pragma("unroll") for (int i_ = (part_) * LPP; i_ < (part_) * LPP + LPP; ++i_) {                            \
            if (i_ < Cfg::A_LOADS)                                                                                  \
                __builtin_amdgcn_global_load_lds((gptr_t)(a_k + (t_).off[i_]),                                      \
                                                 (lptr_t)(sbase + (wave + i_ * Cfg::NW) * 1024), 16, 0, 0);         \
            else                                                                                                    \
                __builtin_amdgcn_global_load_lds((gptr_t)(w_k + (t_).off[i_]),                                      \
                                                 (lptr_t)(sbase + BM * ROW_BYTES + (wave + (i_ - Cfg::A_LOADS) * Cfg::NW) * 1024), 16, 0, 0); \
        }                                                                                                           \
    } while (0)
#define MT_P_FRAGS(buf_, stage_, kk_)                                                                               \
    do {                                                                                                            \
        const unsigned char* sb = lds + (stage_) * Cfg::STAGE_BYTES;                                                \
        _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                             \
            af[buf_][i] = *reinterpret_cast<const bf16x8*>(sb + fa_off[kk_] + i * 32 * ROW_BYTES);                  \
        _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                             \
            wf[buf_][j] = *reinterpret_cast<const bf16x8*>(sb + fw_off[kk_] + j * 32 * ROW_BYTES);                  \
    } while (0)
#define MT_P_MFMAS(buf_)                                                                                            \
    do {                                                                                                            \
        _Pragma("unroll") for (int i = 0; i < TMI; ++i)                                                             \
            _Pragma("unroll") for (int j = 0; j < TNI; ++j)                                                         \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf_][j], af[buf_][i], acc[i][j], 0, 0, 0);  \
    } while (0)

    bf16x8 af[2][TMI], wf[2][TNI];
    f32x16 acc[TMI][TNI];

    // ---- fill: slices 0 .. STAGES-2 of the first tile (KT >= STAGES is a launch condition), then the state every
    //      slice starts in: slice 0 landed for everyone, part 0 of slice STAGES-1 issued, first fragments in registers
#pragma unroll
    for (int p = 0; p < STAGES - 1; ++p) {
#pragma unroll
        for (int part = 0; part < KK; ++part) MT_P_ISSUE(cur, p, p, part);
    }
    p_wait_vmcnt<LPS*(STAGES - 2)>();
    __builtin_amdgcn_s_barrier();
    MT_P_ISSUE(cur, STAGES - 1, STAGES - 1, 0);
    MT_P_FRAGS(0, 0, 0);
    int cs = 0;                                         // ring stage of the slice being multiplied

    // epilogue geometry: a parked row is PARK_COLS float32; on the way out NCH lanes cover a row with 4 columns each
    constexpr int ROWB = Cfg::PARK_ROWB;
    constexpr int NCH = ROWB / 16;
    constexpr int RPW = ROWB >= 256 ? 1 : 256 / ROWB;
    constexpr int ROWS_PER_INST = 64 / NCH;
    constexpr int NIT = 32 / ROWS_PER_INST;
    constexpr int JPB = Cfg::PARK_COLS / 32;                  // 32-column MFMA blocks per parked block
    constexpr int NCB = Cfg::WN / Cfg::PARK_COLS;             // parked blocks across the wavefront's sub-tile
    static_assert(NCH <= 64 && 64 % NCH == 0, "row must split evenly over lanes");
    unsigned char* park = lds + Cfg::RING_BYTES + wave * Cfg::PARK_BYTES;
    const int c = lane % NCH;

    for (int j = 0; j < n_mine; ++j) {
        if (j + 1 < n_mine) locate(j + 1, nxt);
        else nxt = cur;                                 // no next tile: repeat loads of this one, never read
        // this lane's 4 bias values of the tile, fetched now so that the epilogue does not wait for them
        static_assert(NCB == 1, "one parked block across the wavefront's sub-tile");
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        {
            const float* __restrict__ bias = g.bias[cur.grp];
            const int nb = cur.n0 + wn0 + c * 4;
            if (bias && nb < s.N) bv = *reinterpret_cast<const float4*>(bias + nb);
        }
#pragma unroll
        for (int i = 0; i < TMI; ++i)
#pragma unroll
            for (int jj = 0; jj < TNI; ++jj)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

        // One K slice: K steps 0 .. KK-2 read the fragments of the next step and issue the next part of the loads of
        // slice kt+STAGES-1 (tile T1_, slice R1_); the last step follows the sync point (this wavefront's reads of
        // slice kt are in registers, slice kt+1 must have landed for everyone), refills the stage just vacated with
        // part 0 of slice kt+STAGES (tile T0_, slice R0_) and reads the first fragments of slice kt+1.
        // No branch inside: a branch would cut the block the scheduler and the wait-count pass see, and the
        // multiplications of one step would then wait for the fragment reads of the next.
#define MT_P_SLICE(T1_, R1_, T0_, R0_)                                                                              \
        do {                                                                                                        \
            const int ns = cs + 1 == STAGES ? 0 : cs + 1;                                                           \
            const int ps = cs == 0 ? STAGES - 1 : cs - 1;                                                           \
            _Pragma("unroll") for (int kk = 0; kk < KK - 1; ++kk) {                                                 \
                MT_P_FRAGS((kk + 1) & 1, cs, kk + 1);                                                               \
                MT_P_ISSUE(T1_, R1_, ps, kk + 1);                                                                   \
                MT_P_MFMAS(kk & 1);                                                                                 \
                p_interleave<TMI * TNI, TMI + TNI, LPP, MT_P_DSPER>();                                                          \
                __builtin_amdgcn_sched_barrier(0);                                                                  \
            }                                                                                                       \
            p_wait_lgkmcnt0();                                                                                      \
            p_wait_vmcnt<LPS*(STAGES - 2)>();                                                                       \
            __builtin_amdgcn_s_barrier();                                                                           \
            MT_P_ISSUE(T0_, R0_, cs, 0);                                                                            \
            MT_P_FRAGS(0, ns, 0);                                                                                   \
            MT_P_MFMAS((KK - 1) & 1);                                                                               \
            p_interleave<TMI * TNI, TMI + TNI, LPP, MT_P_DSPER>();                                                              \
            __builtin_amdgcn_sched_barrier(0);                                                                      \
            cs = ns;                                                                                                \
        } while (0)
        // slices whose refills still belong to this tile; the one whose second refill is the next tile's slice 0;
        // the last STAGES-1 slices, which fetch the next tile's first slices
        int kt = 0;
        for (; kt < KT - STAGES; ++kt) MT_P_SLICE(cur, kt + STAGES - 1, cur, kt + STAGES);
        MT_P_SLICE(cur, KT - 1, nxt, 0);
        for (kt = 1; kt < STAGES; ++kt) MT_P_SLICE(nxt, kt - 1, nxt, kt);
#undef MT_P_SLICE

        // ---- epilogue of tile `cur`, wavefront-private: park a 32-row x PARK_COLS block of raw accumulators, read ALL of
        //      it back row-contiguously (4 consecutive columns per lane) before touching any of it, so that the LDS
        //      latency is paid once per block, then bias / activation / residual and stores of whole row segments.
        //      Output and residual go through buffer instructions: a row at or beyond M lies at or beyond the buffer's
        //      end and is dropped (stores) or read as zero (loads) by the hardware, and a lane whose columns are beyond N
        //      points beyond the end on purpose; no branch, no 64-bit address arithmetic per row.
        {
            const float* __restrict__ res = g.residual[cur.grp];
            constexpr int ESZ = OUT_F32 ? 4 : 2;
            const uint32_t ldc_b = (uint32_t)s.ldc * ESZ, ldr_b = (uint32_t)s.ldr * 4;
            const __amdgpu_buffer_rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(g.C[cur.grp], 0, (int)((uint32_t)M * ldc_b), 0x00020000);
            const __amdgpu_buffer_rsrc_t r_rs =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(res ? res : (const float*)g.C[cur.grp]), 0, res ? (int)((uint32_t)M * ldr_b) : 0, 0x00020000);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const int n = cur.n0 + wn0 + cb * Cfg::PARK_COLS + c * 4;
                const bool n_ok = n < s.N;                               // N % 4 == 0
                const uint32_t row0 = (uint32_t)(cur.m0 + wm0 + lane / NCH);
                // byte offset of this lane's first row in C / in the residual; 0x80000000 (beyond any buffer) if its columns do not exist
                const uint32_t c_off0 = n_ok ? row0 * ldc_b + (uint32_t)n * ESZ : 0x80000000u;
                const uint32_t r_off0 = n_ok ? row0 * ldr_b + (uint32_t)n * 4 : 0x80000000u;
#pragma unroll
                for (int p = 0; p < TMI; ++p) {
                    // rows of the block are handled GRP at a time (all 8 for bf16 output; 4 for float32 output, where the
                    // residual rows are in registers as well)
                    constexpr int GRP = OUT_F32 ? NIT / 2 : NIT;
                    f32x4 rv[GRP];
                    auto fetch_residual = [&](int it0) {
                        if constexpr (OUT_F32) {
                            if (res) {
#pragma unroll
                                for (int u = 0; u < GRP; ++u)
                                    rv[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                                          r_rs, (int)(r_off0 + (uint32_t)(p * 32 + (it0 + u) * ROWS_PER_INST) * ldr_b), 0, 0));
                            }
                        }
                    };
                    fetch_residual(0);
                    const int key_w = (l32 / RPW) & (NCH - 1);
#pragma unroll
                    for (int jj = 0; jj < JPB; ++jj)
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq) {
                            const int chunk = (jj * 32 + qq * 8 + half * 4) >> 2;
                            const f32x16& a = acc[p][cb * JPB + jj];
                            *reinterpret_cast<float4*>(park + l32 * ROWB + ((chunk ^ key_w) << 4)) =
                                make_float4(a[qq * 4 + 0], a[qq * 4 + 1], a[qq * 4 + 2], a[qq * 4 + 3]);
                        }
                    // the same wavefront reads back what it wrote: LDS operations of one wavefront execute in order
#pragma unroll
                    for (int it0 = 0; it0 < NIT; it0 += GRP) {
                        float4 v[GRP];
#pragma unroll
                        for (int u = 0; u < GRP; ++u) {
                            const int ml = (it0 + u) * ROWS_PER_INST + lane / NCH;
                            const int key = (ml / RPW) & (NCH - 1);
                            v[u] = *reinterpret_cast<const float4*>(park + ml * ROWB + ((c ^ key) << 4));
                        }
#pragma unroll
                        for (int u = 0; u < GRP; ++u) {
                            float4 o;
                            o.x = p_act<ACT>(v[u].x + bv.x);
                            o.y = p_act<ACT>(v[u].y + bv.y);
                            o.z = p_act<ACT>(v[u].z + bv.z);
                            o.w = p_act<ACT>(v[u].w + bv.w);
                            const int off = (int)(c_off0 + (uint32_t)(p * 32 + (it0 + u) * ROWS_PER_INST) * ldc_b);
                            if constexpr (OUT_F32) {
                                if (res) { o.x += rv[u][0]; o.y += rv[u][1]; o.z += rv[u][2]; o.w += rv[u][3]; }
                                const f32x4 ov = {o.x, o.y, o.z, o.w};
                                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, ov), c_rs, off, 0, 0);
                            } else {
                                const bf16x4 ob = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
                                __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, ob), c_rs, off, 0, 0);
                            }
                        }
                        if (it0 + GRP < NIT) fetch_residual(it0 + GRP);
                    }
                }
            }
        }
        cur = nxt;
    }
    // the ring still receives the repeat loads issued past the last tile: they must land before the LDS is released
    p_wait_vmcnt<0>();
#undef MT_P_ISSUE
#undef MT_P_FRAGS
#undef MT_P_MFMAS
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int PARK_COLS, bool OUT_F32, int ACT>
hipError_t p_launch_one(const GemmGroup& g, const GemmShape& s, int n_wg, hipStream_t stream)
{
    using Cfg = PCfg<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS>;
    const int tiles_n = (s.N + BN - 1) / BN;
    auto kfn = gemm_bf16_persist_kernel<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS, OUT_F32, ACT>;
    static std::atomic<uint64_t> lds_raised{0};
    hipError_t e = ensure_dynamic_lds((const void*)kfn, Cfg::LDS_BYTES, lds_raised);
    if (e != hipSuccess) return e;
    // (band heights of 2 .. 16 row-tiles measure the same within noise at these shapes)
    hipLaunchKernelGGL(kfn, dim3(n_wg), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, g, s, tiles_n, kPBand);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int STAGES, int PARK_COLS>
hipError_t p_launch_cfg(const GemmGroup& g, const GemmShape& s, int n_wg, hipStream_t stream)
{
    if (s.out_f32) {
        if (s.act != ACT_NONE) return hipErrorInvalidValue;
        return p_launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS, true, ACT_NONE>(g, s, n_wg, stream);
    }
    switch (s.act) {
        case ACT_NONE: return p_launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS, false, ACT_NONE>(g, s, n_wg, stream);
        case ACT_GELU_ERF: return p_launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS, false, ACT_GELU_ERF>(g, s, n_wg, stream);
        case ACT_GELU_TANH: return p_launch_one<BM, BN, WAVES_M, WAVES_N, BK, STAGES, PARK_COLS, false, ACT_GELU_TANH>(g, s, n_wg, stream);
        default: return hipErrorInvalidValue;
    }
}

// compute units of the current device (cached per device)
int cu_count()
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

bool gemm_bf16_persist_takes(const GemmShape& s)
{
    // K slices must outnumber the ring stages (a tile's refills reach at most into the NEXT tile), no K split,
    // no sub-problems; 32-bit byte offsets as in the tiled kernel
    // (output and residual are addressed through 32-bit buffer offsets with 0x80000000 as the "nowhere" offset)
    if ((uint64_t)s.M * (uint64_t)s.ldc * (s.out_f32 ? 4 : 2) >= (1ull << 31) || (uint64_t)s.M * (uint64_t)s.ldr * 4 >= (1ull << 31)) return false;
    if ((uint64_t)s.M * (uint64_t)s.lda * 2 >= (1ull << 32) || (uint64_t)s.N * (uint64_t)(s.ldw ? s.ldw : s.K) * 2 >= (1ull << 32)) return false;
    return s.splits == 1 && s.n_sub <= 1 && !s.d_sub_rows && s.K % 64 == 0 && s.K / 64 >= 4 && s.N % 4 == 0 &&
           (s.act == ACT_NONE || (!s.out_f32 && (s.act == ACT_GELU_ERF || s.act == ACT_GELU_TANH)));
}

// Rule from measurements at BERT-base and BERT-large widths (1 and 8 problems, 7 k to 20 k rows): with at least one
// 256x256 tile per compute unit the persistent form wins by 5-35 % (most where the output is float32 or K is
// long).  The GELU epilogue is pure vector work that nothing overlaps when one workgroup owns the compute unit, so
// such launches come here only when a part-filled last round of tiles costs little (4 rounds and more by the row
// bound, which over-counts by the padding that is dropped on the device: the rule errs towards the tiled kernel).
bool gemm_bf16_persist_wants(const GemmShape& s)
{
    if (!gemm_bf16_persist_takes(s)) return false;
    const long tiles = (long)s.G * ((s.M + 255) / 256) * ((s.N + 255) / 256);
    const bool gelu = s.act == ACT_GELU_ERF || s.act == ACT_GELU_TANH;
    return tiles >= (long)(gelu ? 4 : 1) * cu_count();
}

hipError_t launch_gemm_bf16_persist(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (!gemm_bf16_persist_takes(s)) return hipErrorInvalidValue;
    const long tiles = (long)s.G * ((s.M + 255) / 256) * ((s.N + 255) / 256);
    const int n_wg = (int)std::min<long>(tiles, cu_count());
    if (n_wg < kPXcds) return hipErrorInvalidValue;          // every XCD's tile range needs a workgroup
    // (rings of two 64-wide and of four 32-wide slices, with a 32 KB park, were measured equal or slower: not instantiated)
    return p_launch_cfg<256, 256, 2, 4, 32, 3, 64>(g, s, n_wg, stream);                       // 96 KB ring, 64 KB park
}

}  // namespace mt
