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

// One K step's instruction mix for the scheduler: NM MFMAs with NF fragment reads and NL global->LDS loads
// slotted between them.
template <int NM, int NF, int NL>
__device__ __forceinline__ void p_interleave()
{
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        else if (i - NF < NL) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
struct PCfg {
    static constexpr int BK = 32, ROW_BYTES = 64, CH = 4, KK = 2, RPI = 16, KEY_SHIFT = 2;
    static constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TMI = WM / 32, TNI = WN / 32;
    static constexpr int A_LOADS = BM / RPI / NW, W_LOADS = BN / RPI / NW, LPS = A_LOADS + W_LOADS;
    static constexpr int LPP = LPS / KK;
    static constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
    static constexpr int RING_BYTES = STAGES * STAGE_BYTES;
    static constexpr int PARK_ROWB = WN * 4;                 // bytes per parked float32 row
    static constexpr int PARK_BYTES = 32 * PARK_ROWB;        // one 32-row block of the wavefront's sub-tile
    static constexpr int LDS_BYTES = RING_BYTES + NW * PARK_BYTES;
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "rows must split evenly over wavefront loads");
    static_assert(LPS % KK == 0, "loads of a slice must split evenly over its K steps");
    static_assert(STAGES >= 3 && LPS * (STAGES - 2) <= 63, "ring depth");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(PARK_ROWB % 256 == 0 || 256 % PARK_ROWB == 0, "park row");
};

// What a workgroup needs to know of one tile to fetch it.
template <int LPS>
struct TileRef {
    const unsigned char* A;
    const unsigned char* W;
    uint32_t off[LPS];     // per load instruction: this lane's byte offset of its 16-byte chunk (row * stride + swizzled chunk)
    int grp, m0, n0;
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool OUT_F32, int ACT>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, 1) void gemm_bf16_persist_kernel(GemmGroup g, GemmShape s, int tiles_n)
{
    using Cfg = PCfg<BM, BN, WAVES_M, WAVES_N, STAGES>;
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

    const int KT = s.K / Cfg::BK;
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
        const int band_sz = kPBand * tiles_n;
        const int band = tt / band_sz;
        const int rows_in_band = min(kPBand, tiles_m - band * kPBand);
        const int tb = tt - band * band_sz;
        const int tn = tb / rows_in_band;
        const int tm = band * kPBand + tb % rows_in_band;
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
    // slice index r of the current tile's K range, or of the next tile's when r runs past it
#define MT_P_ISSUE_AT(r_, stage_, part_)                                                                            \
    do {                                                                                                            \
        if ((r_) < KT) MT_P_ISSUE(cur, (r_), stage_, part_);                                                        \
        else MT_P_ISSUE(nxt, (r_)-KT, stage_, part_);                                                               \
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
        MT_P_ISSUE(cur, p, p, 0);
        MT_P_ISSUE(cur, p, p, 1);
    }
    p_wait_vmcnt<LPS*(STAGES - 2)>();
    __builtin_amdgcn_s_barrier();
    MT_P_ISSUE(cur, STAGES - 1, STAGES - 1, 0);
    MT_P_FRAGS(0, 0, 0);
    int cs = 0;                                         // ring stage of the slice being multiplied

    // epilogue geometry: a parked row is WN float32; on the way out NCH lanes cover a row with 4 columns each
    constexpr int ROWB = Cfg::PARK_ROWB;
    constexpr int NCH = ROWB / 16;
    constexpr int RPW = ROWB >= 256 ? 1 : 256 / ROWB;
    constexpr int ROWS_PER_INST = 64 / NCH;
    constexpr int NIT = 32 / ROWS_PER_INST;
    static_assert(NCH <= 64 && 64 % NCH == 0, "row must split evenly over lanes");
    unsigned char* park = lds + Cfg::RING_BYTES + wave * Cfg::PARK_BYTES;
    const int c = lane % NCH;

    for (int j = 0; j < n_mine; ++j) {
        if (j + 1 < n_mine) locate(j + 1, nxt);
        else nxt = cur;                                 // no next tile: repeat loads of this one, never read
#pragma unroll
        for (int i = 0; i < TMI; ++i)
#pragma unroll
            for (int jj = 0; jj < TNI; ++jj)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

        for (int kt = 0; kt < KT; ++kt) {
            const int ns = cs + 1 == STAGES ? 0 : cs + 1;          // stage of slice kt+1
            const int ps = cs == 0 ? STAGES - 1 : cs - 1;          // stage of slice kt+STAGES-1
            // K step 0: fragments of step 1, second half of the loads of slice kt+STAGES-1
            MT_P_FRAGS(1, cs, 1);
            MT_P_ISSUE_AT(kt + STAGES - 1, ps, 1);
            MT_P_MFMAS(0);
            p_interleave<TMI * TNI, TMI + TNI, LPP>();
            __builtin_amdgcn_sched_barrier(0);
            // sync point: this wavefront's reads of slice kt are in registers, slice kt+1 must have landed
            p_wait_lgkmcnt0();
            p_wait_vmcnt<LPS*(STAGES - 2)>();
            __builtin_amdgcn_s_barrier();
            MT_P_ISSUE_AT(kt + STAGES, cs, 0);                       // stage cs was just vacated by everyone
            MT_P_FRAGS(0, ns, 0);
            MT_P_MFMAS(1);
            p_interleave<TMI * TNI, TMI + TNI, LPP>();
            __builtin_amdgcn_sched_barrier(0);
            cs = ns;
        }

        // ---- epilogue of tile `cur`, wavefront-private: park one 32-row block of raw accumulators, read it back
        //      row-contiguously (4 consecutive columns per lane), bias / activation / residual, store row segments
        const int n = cur.n0 + wn0 + c * 4;
        const bool n_ok = n < s.N;                               // N % 4 == 0
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (g.bias[cur.grp] && n_ok) bv = *reinterpret_cast<const float4*>(g.bias[cur.grp] + n);
        const float* __restrict__ res = g.residual[cur.grp];
        unsigned char* __restrict__ Cout = static_cast<unsigned char*>(g.C[cur.grp]);
        const size_t ldc_b = (size_t)s.ldc * (OUT_F32 ? 4 : 2), ldr_b = (size_t)s.ldr * 4;
#pragma unroll
        for (int p = 0; p < TMI; ++p) {
            const int key_w = (l32 / RPW) & (NCH - 1);
#pragma unroll
            for (int jj = 0; jj < TNI; ++jj)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int chunk = (jj * 32 + qq * 8 + half * 4) >> 2;
                    const f32x16& a = acc[p][jj];
                    *reinterpret_cast<float4*>(park + l32 * ROWB + ((chunk ^ key_w) << 4)) =
                        make_float4(a[qq * 4 + 0], a[qq * 4 + 1], a[qq * 4 + 2], a[qq * 4 + 3]);
                }
            // the same wavefront reads back what it wrote: LDS operations of one wavefront execute in order
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int ml = it * ROWS_PER_INST + lane / NCH;
                const int key = (ml / RPW) & (NCH - 1);
                const float4 v = *reinterpret_cast<const float4*>(park + ml * ROWB + ((c ^ key) << 4));
                const int mm = cur.m0 + wm0 + p * 32 + ml;
                const bool ok = n_ok && mm < M;
                float4 o;
                o.x = p_act<ACT>(v.x + bv.x);
                o.y = p_act<ACT>(v.y + bv.y);
                o.z = p_act<ACT>(v.z + bv.z);
                o.w = p_act<ACT>(v.w + bv.w);
                if constexpr (OUT_F32) {
                    if (res && ok) {
                        const float4 rv = *reinterpret_cast<const float4*>(reinterpret_cast<const unsigned char*>(res) + mm * ldr_b + (size_t)n * 4);
                        o.x += rv.x; o.y += rv.y; o.z += rv.z; o.w += rv.w;
                    }
                    if (ok) *reinterpret_cast<float4*>(Cout + mm * ldc_b + (size_t)n * 4) = o;
                } else {
                    bf16x4 ob = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
                    if (ok) *reinterpret_cast<bf16x4*>(Cout + mm * ldc_b + (size_t)n * 2) = ob;
                }
            }
        }
        cur = nxt;
    }
    // the ring still receives the repeat loads issued past the last tile: they must land before the LDS is released
    p_wait_vmcnt<0>();
#undef MT_P_ISSUE
#undef MT_P_ISSUE_AT
#undef MT_P_FRAGS
#undef MT_P_MFMAS
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool OUT_F32, int ACT>
hipError_t p_launch_one(const GemmGroup& g, const GemmShape& s, int n_wg, hipStream_t stream)
{
    using Cfg = PCfg<BM, BN, WAVES_M, WAVES_N, STAGES>;
    const int tiles_n = (s.N + BN - 1) / BN;
    auto kfn = gemm_bf16_persist_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, OUT_F32, ACT>;
    static std::atomic<uint64_t> lds_raised{0};
    hipError_t e = ensure_dynamic_lds((const void*)kfn, Cfg::LDS_BYTES, lds_raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kfn, dim3(n_wg), dim3(Cfg::NT), Cfg::LDS_BYTES, stream, g, s, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
hipError_t p_launch_cfg(const GemmGroup& g, const GemmShape& s, int n_wg, hipStream_t stream)
{
    if (s.out_f32) {
        if (s.act != ACT_NONE) return hipErrorInvalidValue;
        return p_launch_one<BM, BN, WAVES_M, WAVES_N, STAGES, true, ACT_NONE>(g, s, n_wg, stream);
    }
    switch (s.act) {
        case ACT_NONE: return p_launch_one<BM, BN, WAVES_M, WAVES_N, STAGES, false, ACT_NONE>(g, s, n_wg, stream);
        case ACT_GELU_ERF: return p_launch_one<BM, BN, WAVES_M, WAVES_N, STAGES, false, ACT_GELU_ERF>(g, s, n_wg, stream);
        case ACT_GELU_TANH: return p_launch_one<BM, BN, WAVES_M, WAVES_N, STAGES, false, ACT_GELU_TANH>(g, s, n_wg, stream);
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
    return s.splits == 1 && s.n_sub <= 1 && !s.d_sub_rows && s.K % 32 == 0 && s.K / 32 >= 4 && s.N % 4 == 0 &&
           (s.act == ACT_NONE || (!s.out_f32 && (s.act == ACT_GELU_ERF || s.act == ACT_GELU_TANH)));
}

hipError_t launch_gemm_bf16_persist(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (!gemm_bf16_persist_takes(s)) return hipErrorInvalidValue;
    const long tiles = (long)s.G * ((s.M + 255) / 256) * ((s.N + 255) / 256);
    const int n_wg = (int)std::min<long>(tiles, cu_count());
    if (n_wg < kPXcds) return hipErrorInvalidValue;          // every XCD's tile range needs a workgroup
    return p_launch_cfg<256, 256, 2, 4, 3>(g, s, n_wg, stream);
}

}  // namespace mt
