// Masked-softmax attention, one (problem, sequence, head, 128-query tile) per workgroup.
// A sequence's rows are either its slice of the padding-free row order (seq_start/seq_len given: every
// row is a real token, no mask needed) or the dense rows b*S.. with a key mask.
//
// bfloat16 path (head width 64): the workgroup stages the head's keys K[S][64] and its values,
// transposed to Vt[64][S], in LDS once; each of the 4 wavefronts then owns 32 queries.
// Scores are computed TRANSPOSED, St[key][query] = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then
// holds, for ONE query, 4 consecutive keys per 8-key group, so
//   - a softmax row lives in just two lanes (lane, lane^32): row max and row sum are in-register
//     reductions plus one cross-lane exchange;
//   - the probabilities are already in the register layout of the MFMA's second operand for
//     Ot[d][query] = Vt P^T, so P never goes through LDS;
//   - the per-query rescale of the running output (online softmax over 64-key chunks) and the final
//     1/sum are per-lane scalars.
// Softmax arithmetic is float32 in the log2 domain (exp2 of (score*scale - max)*log2(e)).
// Padding: a masked key gets the score -10000 (selected, not added, so whatever a padded row holds
// cannot leak), its V row is zeroed at staging, and 32-key blocks with no real key are skipped
// altogether (their weights would underflow to exactly zero).  Block 0 is never skipped, so a row
// always has a non-empty softmax.  Wavefronts whose 32 queries are all padding skip their work:
// hidden states at padded positions are unspecified by contract.
//
// float32 path: plain per-query loops for the validation mode, any head width.
#include <type_traits>

#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMaskedScore = -10000.0f;

__device__ inline int k_chunk_off(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

// Two 32-key blocks per online-softmax chunk keep the kernel at 120 registers (four workgroups per compute unit, no
// spills); four blocks per chunk need 158 and measured 5 % slower on 128-token sequences, one block per chunk 1 % faster.
#ifndef MT_ATTN_MINW
#define MT_ATTN_MINW 4
#endif
#ifndef MT_ATTN_CB
#define MT_ATTN_CB 2
#endif
constexpr int CB = MT_ATTN_CB;        // 32-key blocks per online-softmax chunk
__global__ __launch_bounds__(256, MT_ATTN_MINW) void attention_bf16_kernel(AttnGroup g, const int32_t* __restrict__ mask,
                                                             const int32_t* __restrict__ seq_start,
                                                             const int32_t* __restrict__ seq_len, int B, int S, int H, int Sk_max,
                                                             float scale_log2e, int ctx_fmt)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int grp = blockIdx.z / B, b = blockIdx.z % B, a = blockIdx.y;
    const int row0 = seq_start ? seq_start[b] : b * S;             // first row of this sequence
    const int n_tok = seq_len ? min(seq_len[b], S) : S;            // rows (queries and keys) of this sequence
    if ((int)blockIdx.x * 128 >= n_tok) return;                    // whole workgroup: nothing to do
    const int Sk = (n_tok + 31) / 32 * 32;                         // keys rounded up to whole 32-key blocks (<= Sk_max)
    const int vt_stride = Sk + 4;                                  // elements; keeps 8-byte reads aligned, spreads banks
    unsigned char* Ks = lds;                                       // [Sk][128 B], 16-byte chunks XOR-swizzled by row
    __bf16* Vt = reinterpret_cast<__bf16*>(lds + Sk * 128);        // [64][vt_stride]
    float* kvalid = reinterpret_cast<float*>(lds + Sk * 128 + 64 * vt_stride * 2);   // [Sk] 1.0 = real key
    int* blk_any = reinterpret_cast<int*>(kvalid + Sk);            // [Sk/32]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const size_t ld = (size_t)3 * H;
    const __bf16* __restrict__ qkv = static_cast<const __bf16*>(g.qkv[grp]) + (size_t)row0 * ld;
    const int32_t* __restrict__ mrow = mask ? mask + (size_t)b * S : nullptr;
    const int nblk = Sk / 32;

    // ---- this wavefront's 32 queries: their fragments are fetched first, so that the round trip overlaps the staging
    const int q0 = blockIdx.x * 128 + wave * 32;
    const int q = q0 + l32;
    const int qc = q < n_tok ? q : n_tok - 1;
    bf16x8 qf[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8*>(qkv + (size_t)qc * ld + a * 64 + kk * 16 + half * 8);

    // ---- stage K (rows = keys, 8 chunks of 8 elements) and V transposed (item = a pair of adjacent keys x one
    //      8-wide chunk of d).  All of a thread's global loads of a batch are issued before the first LDS write,
    //      so a workgroup pays one memory round trip per batch instead of one per item.
    constexpr int KU = 4, VU = 2;                 // per thread and batch of 128 keys: 4 key chunks, 2 value items
    for (int kb = 0; kb < Sk; kb += 128) {
        uint4 kv[KU], v0[VU], v1[VU];
        int m0[VU], m1[VU];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const int c = kb * 8 + u * 256 + tid;
            const int key = c >> 3, ch = c & 7;
            kv[u] = make_uint4(0, 0, 0, 0);
            if (key < n_tok) kv[u] = *reinterpret_cast<const uint4*>(qkv + (size_t)key * ld + H + a * 64 + ch * 8);
        }
#pragma unroll
        for (int u = 0; u < VU; ++u) {
            const int c = kb * 4 + u * 256 + tid;
            const int pair = c >> 3, ch = c & 7;
            const int k0 = pair * 2, k1 = k0 + 1;
            v0[u] = make_uint4(0, 0, 0, 0);
            v1[u] = make_uint4(0, 0, 0, 0);
            m0[u] = 1;
            m1[u] = 1;
            if (k0 < n_tok) {
                v0[u] = *reinterpret_cast<const uint4*>(qkv + (size_t)k0 * ld + 2 * H + a * 64 + ch * 8);
                if (mrow) m0[u] = mrow[k0];
            }
            if (k1 < n_tok) {
                v1[u] = *reinterpret_cast<const uint4*>(qkv + (size_t)k1 * ld + 2 * H + a * 64 + ch * 8);
                if (mrow) m1[u] = mrow[k1];
            }
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const int c = kb * 8 + u * 256 + tid;
            if ((c >> 3) < Sk) *reinterpret_cast<uint4*>(Ks + k_chunk_off(c >> 3, c & 7)) = kv[u];
        }
#pragma unroll
        for (int u = 0; u < VU; ++u) {
            const int c = kb * 4 + u * 256 + tid;
            const int pair = c >> 3, ch = c & 7;
            const int k0 = pair * 2;
            if (k0 >= Sk) continue;
            if (m0[u] == 0) v0[u] = make_uint4(0, 0, 0, 0);       // a masked key's value row must not leak
            if (m1[u] == 0) v1[u] = make_uint4(0, 0, 0, 0);
            const uint32_t w0[4] = {v0[u].x, v0[u].y, v0[u].z, v0[u].w}, w1[4] = {v1[u].x, v1[u].y, v1[u].z, v1[u].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t lo = (w0[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                const uint32_t hi = (w1[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                *reinterpret_cast<uint32_t*>(Vt + (size_t)(ch * 8 + e) * vt_stride + k0) = lo | (hi << 16);
            }
        }
    }
    // ---- key validity and which 32-key blocks hold a real key
    for (int k = tid; k < Sk; k += 256) kvalid[k] = (k < n_tok && (!mrow || mrow[k] != 0)) ? 1.0f : 0.0f;
    __syncthreads();
    if (tid < nblk) {
        int any = 0;
        for (int k = 0; k < 32; ++k) any |= (kvalid[tid * 32 + k] != 0.0f);
        blk_any[tid] = (tid == 0) ? 1 : any;
    }
    __syncthreads();

    if (q0 >= n_tok) return;
    const bool q_real = (q < n_tok) && (!mrow || mrow[q < n_tok ? q : 0] != 0);
    if (__ballot(q_real) == 0ull) return;

    f32x16 o[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    for (int c0 = 0; c0 < nblk; c0 += CB) {
        int valid[CB];
        int any = 0;
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            valid[j] = (c0 + j < nblk) ? blk_any[c0 + j] : 0;
            any |= valid[j];
        }
        if (!any) continue;
        f32x16 sc[CB];
        float mloc = -INFINITY;
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            if (valid[j]) {
                const int jb = c0 + j;
                f32x16 acc;
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + k_chunk_off(jb * 32 + l32, kk * 2 + half));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], acc, 0, 0, 0);
                }
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const float4 kv = *reinterpret_cast<const float4*>(kvalid + jb * 32 + qq * 8 + half * 4);
                    const float f[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float t = (f[e] != 0.0f) ? acc[qq * 4 + e] * scale_log2e : kMaskedScore * kLog2e;
                        acc[qq * 4 + e] = t;
                        mloc = fmaxf(mloc, t);
                    }
                }
                sc[j] = acc;
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) sc[j][e] = -INFINITY;
            }
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);     // 0 on the first chunk (m_run = -inf)
        float lsum = 0.f;
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(sc[j][e] - m_new);    // bare v_exp_f32: tiny weights flush to 0
                sc[j][e] = p;
                lsum += p;
            }
        lsum += __shfl_xor(lsum, 32, 64);
        l_run = l_run * alpha + lsum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;

#pragma unroll
        for (int j = 0; j < CB; ++j) {
            if (!valid[j]) continue;
            const int jb = c0 + j;
#pragma unroll
            for (int mf = 0; mf < 2; ++mf) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sc[j][mf * 8 + e];
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const __bf16* vrow = Vt + (size_t)(dt * 32 + l32) * vt_stride + jb * 32 + mf * 16 + half * 4;
                    const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vrow);
                    const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vrow + 8);
                    const bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[dt], 0, 0, 0);
                }
            }
        }
    }

    if (q < n_tok && ctx_fmt == 1) {             // E4M3 at unit scale: one byte per element
        const float inv = 1.0f / l_run;
        unsigned char* out = static_cast<unsigned char*>(g.ctx[grp]) + ((size_t)row0 + q) * H + a * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                *reinterpret_cast<uint32_t*>(out + dt * 32 + qq * 8 + half * 4) =
                    pack_e4m3(o[dt][qq * 4 + 0] * inv, o[dt][qq * 4 + 1] * inv, o[dt][qq * 4 + 2] * inv, o[dt][qq * 4 + 3] * inv);
    } else if (q < n_tok) {
        const float inv = 1.0f / l_run;
        __bf16* out = static_cast<__bf16*>(g.ctx[grp]) + ((size_t)row0 + q) * H + a * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                bf16x4 v = {(__bf16)(o[dt][qq * 4 + 0] * inv), (__bf16)(o[dt][qq * 4 + 1] * inv),
                            (__bf16)(o[dt][qq * 4 + 2] * inv), (__bf16)(o[dt][qq * 4 + 3] * inv)};
                *reinterpret_cast<bf16x4*>(out + dt * 32 + qq * 8 + half * 4) = v;
            }
    }
}

// float32 validation path.  One workgroup per (problem, sequence, head); each wavefront takes queries
// wave, wave+4, ...; lanes run over keys for the scores and over head columns for the context.
__global__ __launch_bounds__(256) void attention_f32_kernel(AttnGroup g, const int32_t* __restrict__ mask,
                                                            const int32_t* __restrict__ seq_start,
                                                            const int32_t* __restrict__ seq_len, int B, int Smax, int H, int A,
                                                            float scale)
{
    extern __shared__ float sprob[];   // [4][Smax]
    const int grp = blockIdx.z / B, b = blockIdx.z % B, a = blockIdx.y;
    const int d = H / A;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t ld = (size_t)3 * H;
    const int row0 = seq_start ? seq_start[b] : b * Smax;
    const int S = seq_len ? min(seq_len[b], Smax) : Smax;
    const float* qkv = static_cast<const float*>(g.qkv[grp]) + (size_t)row0 * ld;
    const int32_t* mrow = mask ? mask + (size_t)b * Smax : nullptr;
    float* p = sprob + wave * Smax;
    for (int i = wave; i < S; i += 4) {
        const float* qi = qkv + (size_t)i * ld + a * d;
        float mx = -INFINITY;
        for (int j = lane; j < S; j += 64) {
            const float* kj = qkv + (size_t)j * ld + H + a * d;
            float acc = 0.f;
            for (int c = 0; c < d; ++c) acc = fmaf(qi[c], kj[c], acc);
            float sc = acc * scale;
            if (mrow && mrow[j] == 0) sc += kMaskedScore;
            p[j] = sc;
            mx = fmaxf(mx, sc);
        }
        mx = wave_max(mx);
        float sum = 0.f;
        for (int j = lane; j < S; j += 64) {
            const float e = expf(p[j] - mx);
            p[j] = e;
            sum += e;
        }
        sum = wave_sum(sum);
        const float inv = 1.0f / sum;
        for (int c = lane; c < d; c += 64) {
            float acc = 0.f;
            for (int j = 0; j < S; ++j) acc = fmaf(p[j], qkv[(size_t)j * ld + 2 * H + a * d + c], acc);
            static_cast<float*>(g.ctx[grp])[((size_t)row0 + i) * H + a * d + c] = acc * inv;
        }
    }
}

// First-token query only.  One wavefront per (problem, sequence, head): lanes run over keys for the scores
// (float32 dot product over the head width), the softmax is a wavefront reduction, then lanes run over the
// head's columns for the context.  All of a sequence's rows are real tokens (padding-free row order).
template <typename T>
__global__ __launch_bounds__(64) void attention_cls_kernel(AttnClsGroup g, const int32_t* __restrict__ seq_start,
                                                           const int32_t* __restrict__ seq_len, int B, int Smax, int H, int A,
                                                           float scale)
{
    extern __shared__ float sp[];    // [Smax] scores, then probabilities; then [d] the query
    constexpr int VEC = 16 / (int)sizeof(T);
    const int grp = blockIdx.z / B, b = blockIdx.z % B, a = blockIdx.y;
    const int d = H / A, lane = threadIdx.x;
    const int row0 = seq_start[b];
    const int n = min(seq_len[b], Smax);
    const size_t ld = (size_t)3 * H;
    float* qs = sp + Smax;
    const T* q = static_cast<const T*>(g.q[grp]) + (size_t)b * H + a * d;
    const T* kv = static_cast<const T*>(g.kv[grp]) + (size_t)row0 * ld;
    for (int c = lane; c < d; c += 64) qs[c] = (float)q[c];
    __syncthreads();
    float mx = -INFINITY;
    for (int j = lane; j < n; j += 64) {
        const T* kj = kv + (size_t)j * ld + H + a * d;
        float acc = 0.f;
        if (d % VEC == 0) {                                   // 16-byte loads along the key row
            for (int c = 0; c < d; c += VEC) {
                const uint4 raw = *reinterpret_cast<const uint4*>(kj + c);
                const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
                for (int u = 0; u < VEC; ++u) acc = fmaf(qs[c + u], (float)e[u], acc);
            }
        } else {
            for (int c = 0; c < d; ++c) acc = fmaf(qs[c], (float)kj[c], acc);
        }
        const float sc = acc * scale;
        sp[j] = sc;
        mx = fmaxf(mx, sc);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < n; j += 64) {
        const float e = expf(sp[j] - mx);
        sp[j] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    if (n <= 0) return;
    const float inv = 1.0f / sum;
    for (int c = lane; c < d; c += 64) {                      // lanes over the head's columns: coalesced value rows
        float acc = 0.f;
        const T* vc = kv + 2 * H + a * d + c;
#pragma unroll 4
        for (int j = 0; j < n; ++j) acc = fmaf(sp[j], (float)vc[(size_t)j * ld], acc);
        static_cast<T*>(g.ctx[grp])[(size_t)b * H + a * d + c] = (T)(acc * inv);
    }
}

// Softmax over a sequence's rows of precomputed first-token scores and the probability-weighted sum of the
// layer input rows, per head (see PoolGroup).  One workgroup per (problem, sequence, 256-column slab); every
// workgroup repeats the (tiny) softmax, then each thread owns one column of the slab for all heads.
constexpr int kPoolMaxHeads = 16;
template <int NA4>      // A_pad / 4: compile-time head count keeps the accumulators and the probability reads branch-free
__global__ __launch_bounds__(256) void first_token_pool_kernel(PoolGroup g, const int32_t* __restrict__ seq_start,
                                                               const int32_t* __restrict__ seq_len, int B, int Smax, int H, int A,
                                                               int A_pad, float scale)
{
    extern __shared__ float pl[];                       // [Smax][A_pad] scores, then probabilities
    const int grp = blockIdx.y, b = blockIdx.x;
    const int row0 = seq_start[b];
    const int n = min(seq_len[b], Smax);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* __restrict__ sc = g.scores[grp] + (size_t)row0 * A_pad;
    for (int i0 = 0; i0 < n * A_pad; i0 += 256 * 8) {      // all of a thread's loads of a batch are in flight together
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * 256 + tid;
            v[u] = i < n * A_pad ? sc[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * 256 + tid;
            if (i < n * A_pad) pl[i] = v[u] * scale;
        }
    }
    __syncthreads();
    for (int a = wave; a < A; a += 4) {                 // one head per wavefront at a time, lanes over keys
        float mx = -INFINITY;
        for (int j = lane; j < n; j += 64) mx = fmaxf(mx, pl[j * A_pad + a]);
        mx = wave_max(mx);
        float sum = 0.f;
        for (int j = lane; j < n; j += 64) {
            const float e = expf(pl[j * A_pad + a] - mx);
            pl[j * A_pad + a] = e;
            sum += e;
        }
        sum = wave_sum(sum);
        const float inv = 1.0f / sum;
        for (int j = lane; j < n; j += 64) pl[j * A_pad + a] *= inv;
    }
    __syncthreads();
    // every thread owns TWO adjacent columns (4-byte loads: sub-dword loads issue no faster than dword ones)
    const int c = (blockIdx.z * 256 + tid) * 2;
    if (c >= H || n <= 0) return;
    float acc[NA4 * 4][2];
#pragma unroll
    for (int a = 0; a < NA4 * 4; ++a) acc[a][0] = acc[a][1] = 0.f;
    const __bf16* __restrict__ x = static_cast<const __bf16*>(g.x[grp]) + (size_t)row0 * H + c;
    // rows in batches of JU: the batch's row loads and probability reads are all issued before the first FMA
    constexpr int JU = 8;
    auto rows = [&](int j0, auto full) {
        bf16x2 xv[JU];
        float4 p4[JU][NA4];
#pragma unroll
        for (int u = 0; u < JU; ++u)
            if (full || j0 + u < n) xv[u] = *reinterpret_cast<const bf16x2*>(x + (size_t)(j0 + u) * H);
#pragma unroll
        for (int u = 0; u < JU; ++u)
            if (full || j0 + u < n) {
#pragma unroll
                for (int a4 = 0; a4 < NA4; ++a4) p4[u][a4] = *reinterpret_cast<const float4*>(pl + (j0 + u) * A_pad + a4 * 4);   // broadcast
            }
#pragma unroll
        for (int u = 0; u < JU; ++u)
            if (full || j0 + u < n) {
                const float x0 = (float)xv[u][0], x1 = (float)xv[u][1];
#pragma unroll
                for (int a4 = 0; a4 < NA4; ++a4) {
                    acc[a4 * 4 + 0][0] = fmaf(p4[u][a4].x, x0, acc[a4 * 4 + 0][0]);
                    acc[a4 * 4 + 0][1] = fmaf(p4[u][a4].x, x1, acc[a4 * 4 + 0][1]);
                    acc[a4 * 4 + 1][0] = fmaf(p4[u][a4].y, x0, acc[a4 * 4 + 1][0]);
                    acc[a4 * 4 + 1][1] = fmaf(p4[u][a4].y, x1, acc[a4 * 4 + 1][1]);
                    acc[a4 * 4 + 2][0] = fmaf(p4[u][a4].z, x0, acc[a4 * 4 + 2][0]);
                    acc[a4 * 4 + 2][1] = fmaf(p4[u][a4].z, x1, acc[a4 * 4 + 2][1]);
                    acc[a4 * 4 + 3][0] = fmaf(p4[u][a4].w, x0, acc[a4 * 4 + 3][0]);
                    acc[a4 * 4 + 3][1] = fmaf(p4[u][a4].w, x1, acc[a4 * 4 + 3][1]);
                }
            }
    };
    int j0 = 0;
    for (; j0 + JU <= n; j0 += JU) rows(j0, std::true_type{});
    if (j0 < n) rows(j0, std::false_type{});
    __bf16* out = static_cast<__bf16*>(g.xbar[grp]) + (size_t)b * A_pad * H + c;
#pragma unroll
    for (int a = 0; a < NA4 * 4; ++a)
        if (a < A) {
            const bf16x2 o = {(__bf16)acc[a][0], (__bf16)acc[a][1]};
            *reinterpret_cast<bf16x2*>(out + (size_t)a * H) = o;
        }
}

}  // namespace

hipError_t launch_first_token_pool(const PoolGroup& g, int G, const int32_t* seq_start, const int32_t* seq_len, int B, int S, int H,
                                   int A, int A_pad, hipStream_t stream)
{
    if (G <= 0 || B <= 0 || S <= 0) return hipSuccess;
    if (!seq_start || !seq_len || G > kMaxGroup || A < 1 || A > kPoolMaxHeads || A_pad < A || A_pad > kPoolMaxHeads || A_pad % 4 != 0 || H % 2 != 0 ||
        (size_t)S * A_pad * 4 > 64 * 1024)
        return hipErrorInvalidValue;
    dim3 grid(B, G, (H + 511) / 512), block(256);
    const size_t lds = (size_t)S * A_pad * sizeof(float);
    const float scale = 1.0f / sqrtf((float)(H / A));
    switch (A_pad / 4) {
        case 1: hipLaunchKernelGGL(first_token_pool_kernel<1>, grid, block, lds, stream, g, seq_start, seq_len, B, S, H, A, A_pad, scale); break;
        case 2: hipLaunchKernelGGL(first_token_pool_kernel<2>, grid, block, lds, stream, g, seq_start, seq_len, B, S, H, A, A_pad, scale); break;
        case 3: hipLaunchKernelGGL(first_token_pool_kernel<3>, grid, block, lds, stream, g, seq_start, seq_len, B, S, H, A, A_pad, scale); break;
        default: hipLaunchKernelGGL(first_token_pool_kernel<4>, grid, block, lds, stream, g, seq_start, seq_len, B, S, H, A, A_pad, scale); break;
    }
    return hipGetLastError();
}

hipError_t launch_attention_cls(const AttnClsGroup& g, int G, int is_bf16, const int32_t* seq_start, const int32_t* seq_len,
                                int B, int S, int H, int A, hipStream_t stream)
{
    if (G <= 0 || B <= 0 || S <= 0) return hipSuccess;
    if (!seq_start || !seq_len || G > kMaxGroup || H % A != 0 || ((size_t)S + H / A) * 4 > 64 * 1024) return hipErrorInvalidValue;
    dim3 grid(1, A, B * G), block(64);
    const float scale = 1.0f / sqrtf((float)(H / A));
    if (is_bf16)
        hipLaunchKernelGGL((attention_cls_kernel<__bf16>), grid, block, ((size_t)S + H / A) * sizeof(float), stream, g, seq_start, seq_len, B, S, H,
                           A, scale);
    else
        hipLaunchKernelGGL((attention_cls_kernel<float>), grid, block, ((size_t)S + H / A) * sizeof(float), stream, g, seq_start, seq_len, B, S, H,
                           A, scale);
    return hipGetLastError();
}

hipError_t launch_attention_bf16(const AttnGroup& g, int G, const int32_t* mask, const int32_t* seq_start,
                                 const int32_t* seq_len, int B, int S, int H, int A, hipStream_t stream, int ctx_fmt)
{
    if (!mask && !(seq_start && seq_len)) return hipErrorInvalidValue;
    if (G <= 0 || B <= 0 || S <= 0) return hipSuccess;
    if (H != A * 64 || G > kMaxGroup || S > kAttnBf16MaxSeq || (ctx_fmt != 0 && ctx_fmt != 1)) return hipErrorInvalidValue;
    const int Sk = (S + 31) / 32 * 32;
    const size_t lds = (size_t)Sk * 128 + (size_t)64 * (Sk + 4) * 2 + (size_t)Sk * 4 + (size_t)(Sk / 32) * 4;
    static_assert(kAttnBf16MaxSeq % 32 == 0 &&
                      (size_t)kAttnBf16MaxSeq * 128 + (size_t)64 * (kAttnBf16MaxSeq + 4) * 2 + (size_t)kAttnBf16MaxSeq * 4 +
                              (size_t)(kAttnBf16MaxSeq / 32) * 4 <= 160 * 1024 &&
                      (size_t)(kAttnBf16MaxSeq + 32) * 260 + 512 > 160 * 1024,
                  "kAttnBf16MaxSeq is the largest multiple of 32 whose keys and values fit the LDS");
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    static std::atomic<uint64_t> lds_raised{0};
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)attention_bf16_kernel, 160 * 1024, lds_raised);
        if (e != hipSuccess) return e;
    }
    dim3 grid((S + 127) / 128, A, B * G), block(256);
    const float scale_log2e = (1.0f / sqrtf(64.0f)) * kLog2e;
    hipLaunchKernelGGL(attention_bf16_kernel, grid, block, lds, stream, g, mask, seq_start, seq_len, B, S, H, Sk, scale_log2e, ctx_fmt);
    return hipGetLastError();
}

hipError_t launch_attention_f32(const AttnGroup& g, int G, const int32_t* mask, const int32_t* seq_start,
                                const int32_t* seq_len, int B, int S, int H, int A, hipStream_t stream)
{
    if (!mask && !(seq_start && seq_len)) return hipErrorInvalidValue;
    if (G <= 0 || B <= 0 || S <= 0) return hipSuccess;
    if (G > kMaxGroup || (size_t)S * 16 > 64 * 1024) return hipErrorInvalidValue;
    dim3 grid(1, A, B * G), block(256);
    const float scale = 1.0f / sqrtf((float)(H / A));
    hipLaunchKernelGGL(attention_f32_kernel, grid, block, (size_t)S * 4 * sizeof(float), stream, g, mask, seq_start, seq_len, B, S, H, A,
                       scale);
    return hipGetLastError();
}

}  // namespace mt
