// Row kernels: the padding-free row map, embedding sum + LayerNorm, LayerNorm of a pre-summed row,
// pooler input split and classifier.
// One 64-lane wavefront owns one row; statistics are float32 with a two-pass variance taken from
// registers, reductions are wavefront shuffles.  Both kernels are HBM-bound: each row is read once
// and written once (float32 and, for the matrix-core path, a bfloat16 copy).
#include <algorithm>

#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int kRowsPerBlock = 4;   // 4 wavefronts of 64 lanes

template <typename T>
__device__ inline float4 load4(const T* p);
template <>
__device__ inline float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <>
__device__ inline float4 load4<__bf16>(const __bf16* p)
{
    bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}

// Normalise NV float4 per lane held in registers and store.  gamma and beta arrive in registers: their loads are issued
// with the row's, ahead of the two reductions.
template <int NV>
__device__ inline void ln_finish_store(float4 (&v)[NV], const float4 (&g)[NV], const float4 (&b)[NV], int lane, int H, float eps,
                                       float* out_f32, __bf16* out_bf16, int low_fmt = 0)
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    const float mean = wave_sum(s) / (float)H;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float a = v[i].x - mean, bb = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
        q += (a * a + bb * bb) + (c * c + d * d);
    }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)H + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int col = (i * 64 + lane) * 4;
        float4 o;
        o.x = g[i].x * ((v[i].x - mean) * inv) + b[i].x;
        o.y = g[i].y * ((v[i].y - mean) * inv) + b[i].y;
        o.z = g[i].z * ((v[i].z - mean) * inv) + b[i].z;
        o.w = g[i].w * ((v[i].w - mean) * inv) + b[i].w;
        if (out_f32) *reinterpret_cast<float4*>(out_f32 + col) = o;
        if (out_bf16 && low_fmt == 1) {                   // E4M3, one byte per element
            *reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(out_bf16) + col) = pack_e4m3(o.x, o.y, o.z, o.w);
        } else if (out_bf16) {
            bf16x4 p = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
            *reinterpret_cast<bf16x4*>(out_bf16 + col) = p;
        }
    }
}

template <int NV>
__device__ inline void ln_load_gamma_beta(const float* gamma, const float* beta, int lane, float4 (&g)[NV], float4 (&b)[NV])
{
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int col = (i * 64 + lane) * 4;
        g[i] = *reinterpret_cast<const float4*>(gamma + col);
        b[i] = *reinterpret_cast<const float4*>(beta + col);
    }
}

// H == NV*256: the whole row lives in registers.  All of a lane's loads (row, residual, bias, gamma, beta: 5 NV
// 16-byte loads) are issued before the first use, in blocks without uses of their own, so that a wavefront pays one
// memory round trip per row (loads guarded one by one, each followed by its add, were waited for one at a time).
template <int NV>
__global__ __launch_bounds__(256) void layernorm_fast(LnGroup g, int M, const int32_t* __restrict__ d_M, int H, float eps,
                                                      int n_parts, int64_t part_stride, int low_fmt)
{
    const int grp = blockIdx.y;
    const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (d_M) M = min(M, *d_M);
    if (row >= M) return;
    const float* x = g.x[grp] + (size_t)row * H;
    const float* res = g.residual[grp] ? g.residual[grp] + (size_t)row * H : nullptr;
    const float* bias = g.bias[grp];
    float4 v[NV], rv[NV], bv[NV], gm[NV], bt[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = *reinterpret_cast<const float4*>(x + (i * 64 + lane) * 4);
    if (res) {
#pragma unroll
        for (int i = 0; i < NV; ++i) rv[i] = *reinterpret_cast<const float4*>(res + (i * 64 + lane) * 4);
    } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) rv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (bias) {
#pragma unroll
        for (int i = 0; i < NV; ++i) bv[i] = *reinterpret_cast<const float4*>(bias + (i * 64 + lane) * 4);
    } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) bv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    ln_load_gamma_beta<NV>(g.gamma[grp], g.beta[grp], lane, gm, bt);
    __builtin_amdgcn_sched_barrier(0);
    for (int p = 1; p < n_parts; ++p) {                           // fixed order: deterministic
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const float4 t = *reinterpret_cast<const float4*>(x + (size_t)p * part_stride + (i * 64 + lane) * 4);
            v[i].x += t.x; v[i].y += t.y; v[i].z += t.z; v[i].w += t.w;
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {                                // (sum of partial products + bias) + residual, as before
        v[i].x = (v[i].x + bv[i].x) + rv[i].x;
        v[i].y = (v[i].y + bv[i].y) + rv[i].y;
        v[i].z = (v[i].z + bv[i].z) + rv[i].z;
        v[i].w = (v[i].w + bv[i].w) + rv[i].w;
    }
    float* of = g.out_f32[grp] ? g.out_f32[grp] + (size_t)row * H : nullptr;
    // the low-precision copy's row is H elements of 2 bytes (bf16) or 1 byte (E4M3)
    __bf16* ob = g.out_bf16[grp] ? reinterpret_cast<__bf16*>(reinterpret_cast<unsigned char*>(g.out_bf16[grp]) + (size_t)row * H * (low_fmt == 1 ? 1 : 2))
                                 : nullptr;
    ln_finish_store<NV>(v, gm, bt, lane, H, eps, of, ob, low_fmt);
}

// Any H: three strided passes over the row (it stays in cache between passes).
__global__ __launch_bounds__(256) void layernorm_any(LnGroup g, int M, const int32_t* __restrict__ d_M, int H, float eps,
                                                     int n_parts, int64_t part_stride, int low_fmt)
{
    const int grp = blockIdx.y;
    const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (d_M) M = min(M, *d_M);
    if (row >= M) return;
    const float* xp = g.x[grp] + (size_t)row * H;
    const float* res = g.residual[grp] ? g.residual[grp] + (size_t)row * H : nullptr;
    const float* bias = g.bias[grp];
    auto value = [&](int i) {
        float t = xp[i];
        for (int p = 1; p < n_parts; ++p) t += xp[(size_t)p * part_stride + i];
        if (bias) t += bias[i];
        if (res) t += res[i];
        return t;
    };
    float s = 0.f;
    for (int i = lane; i < H; i += 64) s += value(i);
    const float mean = wave_sum(s) / (float)H;
    float q = 0.f;
    for (int i = lane; i < H; i += 64) { float d = value(i) - mean; q += d * d; }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)H + eps);
    const float* gamma = g.gamma[grp];
    const float* beta = g.beta[grp];
    float* of = g.out_f32[grp] ? g.out_f32[grp] + (size_t)row * H : nullptr;
    __bf16* ob = g.out_bf16[grp] ? reinterpret_cast<__bf16*>(g.out_bf16[grp]) + (size_t)row * H : nullptr;
    unsigned char* o8 = g.out_bf16[grp] ? reinterpret_cast<unsigned char*>(g.out_bf16[grp]) + (size_t)row * H : nullptr;
    for (int i = lane; i < H; i += 64) {
        float o = gamma[i] * ((value(i) - mean) * inv) + beta[i];
        if (of) of[i] = o;
        if (ob && low_fmt == 1) o8[i] = (unsigned char)(pack_e4m3(o, 0.f, 0.f, 0.f) & 0xFFu);
        else if (ob) ob[i] = (__bf16)o;
    }
}

template <typename TE, int NV>
__global__ __launch_bounds__(256) void embed_ln_fast(const int32_t* ids, const int32_t* __restrict__ type_ids, int type_vocab, const int32_t* __restrict__ src,
                                                     const int32_t* __restrict__ d_M, int M, int S, int H, int vocab,
                                                     const TE* word, const TE* pos, const TE* type,
                                                     const float* gamma, const float* beta, float eps,
                                                     float* out_f32, __bf16* out_bf16)
{
    const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (d_M) M = min(M, *d_M);
    if (row >= M) return;
    const int p_idx = src ? src[row] : row;
    int id = ids[p_idx];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const int s = p_idx % S;
    int seg = type_ids ? type_ids[p_idx] : 0;
    seg = seg < 0 ? 0 : (seg >= type_vocab ? type_vocab - 1 : seg);
    type += (size_t)seg * H;
    const TE* w = word + (size_t)id * H;
    const TE* p = pos + (size_t)s * H;
    float4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int col = (i * 64 + lane) * 4;
        float4 a = load4<TE>(w + col), b = load4<TE>(p + col), c = load4<TE>(type + col);
        v[i] = make_float4((a.x + b.x) + c.x, (a.y + b.y) + c.y, (a.z + b.z) + c.z, (a.w + b.w) + c.w);
    }
    float4 gm[NV], bt[NV];
    ln_load_gamma_beta<NV>(gamma, beta, lane, gm, bt);
    ln_finish_store<NV>(v, gm, bt, lane, H, eps, out_f32 ? out_f32 + (size_t)row * H : nullptr,
                        out_bf16 ? out_bf16 + (size_t)row * H : nullptr);
}

template <typename TE>
__global__ __launch_bounds__(256) void embed_ln_any(const int32_t* ids, const int32_t* __restrict__ type_ids, int type_vocab, const int32_t* __restrict__ src,
                                                    const int32_t* __restrict__ d_M, int M, int S, int H, int vocab,
                                                    const TE* word, const TE* pos, const TE* type,
                                                    const float* gamma, const float* beta, float eps,
                                                    float* out_f32, __bf16* out_bf16)
{
    const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (d_M) M = min(M, *d_M);
    if (row >= M) return;
    const int p_idx = src ? src[row] : row;
    int id = ids[p_idx];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const int sidx = p_idx % S;
    int seg = type_ids ? type_ids[p_idx] : 0;
    seg = seg < 0 ? 0 : (seg >= type_vocab ? type_vocab - 1 : seg);
    type += (size_t)seg * H;
    const TE* w = word + (size_t)id * H;
    const TE* p = pos + (size_t)sidx * H;
    float s = 0.f;
    for (int i = lane; i < H; i += 64) s += ((float)w[i] + (float)p[i]) + (float)type[i];
    const float mean = wave_sum(s) / (float)H;
    float q = 0.f;
    for (int i = lane; i < H; i += 64) {
        float d = ((float)w[i] + (float)p[i]) + (float)type[i] - mean;
        q += d * d;
    }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)H + eps);
    for (int i = lane; i < H; i += 64) {
        float e = ((float)w[i] + (float)p[i]) + (float)type[i];
        float o = gamma[i] * ((e - mean) * inv) + beta[i];
        if (out_f32) out_f32[(size_t)row * H + i] = o;
        if (out_bf16) out_bf16[(size_t)row * H + i] = (__bf16)o;
    }
}

template <typename TE>
hipError_t embed_dispatch(const int32_t* ids, const int32_t* type_ids, int type_vocab, const int32_t* src, const int32_t* d_M, int B, int S, int H, int vocab, const TE* word, const TE* pos,
                          const TE* type, const float* gamma, const float* beta, float eps, float* of, __bf16* ob,
                          hipStream_t st)
{
    const int M = B * S;
    dim3 grid((M + kRowsPerBlock - 1) / kRowsPerBlock), block(256);
    if (H == 768)
        hipLaunchKernelGGL((embed_ln_fast<TE, 3>), grid, block, 0, st, ids, type_ids, type_vocab, src, d_M, M, S, H, vocab, word, pos, type, gamma, beta, eps, of, ob);
    else if (H == 1024)
        hipLaunchKernelGGL((embed_ln_fast<TE, 4>), grid, block, 0, st, ids, type_ids, type_vocab, src, d_M, M, S, H, vocab, word, pos, type, gamma, beta, eps, of, ob);
    else if (H == 256)
        hipLaunchKernelGGL((embed_ln_fast<TE, 1>), grid, block, 0, st, ids, type_ids, type_vocab, src, d_M, M, S, H, vocab, word, pos, type, gamma, beta, eps, of, ob);
    else if (H == 512)
        hipLaunchKernelGGL((embed_ln_fast<TE, 2>), grid, block, 0, st, ids, type_ids, type_vocab, src, d_M, M, S, H, vocab, word, pos, type, gamma, beta, eps, of, ob);
    else
        hipLaunchKernelGGL((embed_ln_any<TE>), grid, block, 0, st, ids, type_ids, type_vocab, src, d_M, M, S, H, vocab, word, pos, type, gamma, beta, eps, of, ob);
    return hipGetLastError();
}

// Pass 1 of the row map, one workgroup per sequence: rank of every real token inside its sequence
// (written into row_of, -1 for padding) and the sequence's count of real tokens.
__global__ __launch_bounds__(256) void row_rank_kernel(const int32_t* __restrict__ mask, int S, int32_t* __restrict__ row_of,
                                                       int32_t* __restrict__ seq_len)
{
    __shared__ int wave_cnt[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = 0;
    for (int c0 = 0; c0 < S; c0 += 256) {
        const int s = c0 + tid;
        const bool flag = s < S && mask[(size_t)b * S + s] != 0;
        const unsigned long long bal = __ballot(flag);
        const int lane_rank = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int woff = 0, total = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) woff += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (s < S) row_of[(size_t)b * S + s] = flag ? base + woff + lane_rank : -1;
        base += total;
        __syncthreads();
    }
    if (tid == 0) seq_len[b] = base;
}

// Pass 2: sequence b starts at the sum of the counts before it; ranks become global rows.
__global__ __launch_bounds__(256) void row_place_kernel(int B, int S, int32_t* __restrict__ row_of,
                                                        const int32_t* __restrict__ seq_len, int32_t* __restrict__ seq_start,
                                                        int32_t* __restrict__ src, int32_t* __restrict__ n_rows)
{
    __shared__ int part[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int acc = 0;
    for (int i = tid; i < b; i += 256) acc += seq_len[i];
    acc = wave_sum_int(acc);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    const int start = part[0] + part[1] + part[2] + part[3];
    if (tid == 0) {
        seq_start[b] = start;
        if (b == B - 1) *n_rows = start + seq_len[b];
    }
    for (int s = tid; s < S; s += 256) {
        const size_t p = (size_t)b * S + s;
        const int r = row_of[p];
        if (r >= 0) {
            row_of[p] = start + r;
            src[start + r] = (int)p;
        }
    }
}

__global__ __launch_bounds__(256) void unpack_rows_kernel(const float* __restrict__ x, const int32_t* __restrict__ row_of, int n_pos,
                                                          int H, float* __restrict__ out)
{
    const int p = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (p >= n_pos) return;
    const int r = row_of[p];
    for (int i = lane; i < H; i += 64) out[(size_t)p * H + i] = r >= 0 ? x[(size_t)r * H + i] : 0.f;
}

__global__ __launch_bounds__(256) void cls_split_kernel(SplitGroup g, int H, const int32_t* __restrict__ seq_start,
                                                        int rows_per_seq, int max_rows)
{
    const int grp = blockIdx.y, b = blockIdx.x;
    const int row = g.compact[grp] ? b : min(seq_start ? seq_start[b] : b * rows_per_seq, max_rows - 1);
    const float* x = g.x[grp] + (size_t)row * H;
    __bf16* out = reinterpret_cast<__bf16*>(g.out[grp]) + (size_t)b * 2 * H;
    for (int i = threadIdx.x; i < H; i += 256) {
        const float v = x[i];
        const __bf16 hi = (__bf16)v;
        out[i] = hi;
        out[H + i] = (__bf16)(v - (float)hi);
    }
}

__global__ __launch_bounds__(256) void gather_rows_kernel(SplitGroup g, int H, const int32_t* __restrict__ seq_start,
                                                          int rows_per_seq, int max_rows)
{
    const int grp = blockIdx.y, b = blockIdx.x;
    const int row = g.compact[grp] ? b : min(seq_start ? seq_start[b] : b * rows_per_seq, max_rows - 1);
    const float* x = g.x[grp] + (size_t)row * H;
    float* out = reinterpret_cast<float*>(g.out[grp]) + (size_t)b * H;
    for (int i = threadIdx.x; i < H; i += 256) out[i] = x[i];
}

__global__ __launch_bounds__(256) void gather_first_rows_kernel(FirstRowsGroup g, int H, int act_bytes,
                                                                const int32_t* __restrict__ seq_start, int max_rows)
{
    const int grp = blockIdx.y, b = blockIdx.x;
    const int row = min(seq_start[b], max_rows - 1);
    if (g.xf[grp]) {
        const float* x = g.xf[grp] + (size_t)row * H;
        float* o = g.out_f[grp] + (size_t)b * H;
        for (int i = threadIdx.x; i < H; i += 256) o[i] = x[i];
    }
    if (g.xa[grp]) {
        const size_t nbytes = (size_t)H * act_bytes;            // H * 2 or H * 4, a multiple of 4 (H is even in bf16 mode)
        const uint32_t* x = reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(g.xa[grp]) + (size_t)row * nbytes);
        uint32_t* o = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(g.out_a[grp]) + (size_t)b * nbytes);
        for (int i = threadIdx.x; i < (int)(nbytes / 4); i += 256) o[i] = x[i];
    }
}

__global__ __launch_bounds__(256) void place_first_rows_kernel(const float* __restrict__ x, int n_pos, int S, int H,
                                                               float* __restrict__ out)
{
    const int p = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (p >= n_pos) return;
    const bool first = (p % S) == 0;
    const float* src = x + (size_t)(p / S) * H;
    for (int i = lane; i < H; i += 64) out[(size_t)p * H + i] = first ? src[i] : 0.f;
}

template <typename TW>
__global__ __launch_bounds__(256) void classifier_kernel(ClsGroup g, int B, int H, int64_t ldo, const int32_t* __restrict__ out_row)
{
    const int grp = blockIdx.y, b = blockIdx.x;
    const int ob = out_row ? out_row[b] : b;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* p = g.pooled[grp] + (size_t)b * H;
    const int c = blockIdx.z * 4 + wave;            // one wavefront per class
    if (c >= g.C[grp]) return;
    const TW* w = static_cast<const TW*>(g.Wc[grp]) + (size_t)c * H;
    float acc = 0.f;
    for (int i = lane; i < H; i += 64) acc = fmaf(p[i], (float)w[i], acc);
    acc = wave_sum(acc);
    if (lane == 0) g.out[grp][(size_t)ob * ldo + c] = acc + g.bc[grp][c];
}

// Token-level head.  A workgroup owns 16 consecutive positions, each of its 4 wavefronts 4 of them, so that a row
// of Wc is fetched once per 4 positions; lanes stride over the hidden dimension, float32 accumulation.
constexpr int kTokPosPerWave = 4;
constexpr int kRowSkip = -2;          // row_of value: the position belongs to no sequence of this launch (see launch_route_rowof)
template <typename TW>
__global__ __launch_bounds__(256) void token_classifier_kernel(TokGroup g, int n_pos, int H, int64_t ldo,
                                                               const int32_t* __restrict__ row_of,
                                                               const int32_t* __restrict__ n_rows)
{
    const int grp = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p0 = (blockIdx.x * 4 + wave) * kTokPosPerWave;
    if (p0 >= n_pos) return;
    const int kept = *n_rows;
    const int C = g.C[grp];
    const float* xr[kTokPosPerWave];
    bool live[kTokPosPerWave], skip[kTokPosPerWave];
#pragma unroll
    for (int j = 0; j < kTokPosPerWave; ++j) {
        const int p = p0 + j;
        const int r = p < n_pos ? row_of[p] : kRowSkip;
        live[j] = r >= 0 && r < kept;
        skip[j] = r == kRowSkip;
        xr[j] = g.x[grp] + (size_t)(live[j] ? r : 0) * H;
    }
    const bool any = live[0] || live[1] || live[2] || live[3];
    for (int c = 0; c < C; ++c) {
        float acc[kTokPosPerWave] = {0.f, 0.f, 0.f, 0.f};
        if (any) {
            const TW* w = static_cast<const TW*>(g.Wc[grp]) + (size_t)c * H;
            for (int i = lane; i < H; i += 64) {
                const float wv = (float)w[i];
#pragma unroll
                for (int j = 0; j < kTokPosPerWave; ++j) acc[j] = fmaf(live[j] ? xr[j][i] : 0.f, wv, acc[j]);
            }
        }
        const float bias = g.bc[grp][c];
#pragma unroll
        for (int j = 0; j < kTokPosPerWave; ++j) {
            const float v = wave_sum(acc[j]);
            if (lane == 0 && !skip[j]) g.out[grp][(size_t)(p0 + j) * ldo + c] = live[j] ? v + bias : 0.f;
        }
    }
}

// The same for H = NV * 256: one wavefront per position keeps its row in registers (NV float4 per lane) and takes
// the classes four at a time, so the loads of four weight rows are in flight together.
template <typename TW, int NV>
__global__ __launch_bounds__(256) void token_classifier_rows_kernel(TokGroup g, int n_pos, int64_t ldo,
                                                                    const int32_t* __restrict__ row_of,
                                                                    const int32_t* __restrict__ n_rows)
{
    constexpr int H = NV * 256;
    const int grp = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= n_pos) return;
    const int C = g.C[grp];
    float* out = g.out[grp] + (size_t)p * ldo;
    const int r = row_of[p];
    if (r == kRowSkip) return;                        // not this launch's position: left untouched
    if (r < 0 || r >= *n_rows) {
        for (int c = lane; c < C; c += 64) out[c] = 0.f;
        return;
    }
    const float* x = g.x[grp] + (size_t)r * H;
    float4 xv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) xv[v] = load4<float>(x + (v * 64 + lane) * 4);
    const TW* W = static_cast<const TW*>(g.Wc[grp]);
    for (int c0 = 0; c0 < C; c0 += 4) {
        float acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const TW* w = W + (size_t)min(c0 + u, C - 1) * H;
            float a = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float4 wv = load4<TW>(w + (v * 64 + lane) * 4);
                a = fmaf(xv[v].x, wv.x, a);
                a = fmaf(xv[v].y, wv.y, a);
                a = fmaf(xv[v].z, wv.z, a);
                a = fmaf(xv[v].w, wv.w, a);
            }
            acc[u] = a;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float v = wave_sum(acc[u]);
            if (lane == 0 && c0 + u < C) out[c0 + u] = v + g.bc[grp][c0 + u];
        }
    }
}

// Row order of a sub-batch (per-sequence routing).  One workgroup: lengths of the chosen sequences, their prefix
// sums (n_sel <= 1024, four per thread), then for every chosen sequence the batch rows its compact rows copy.
__global__ __launch_bounds__(256) void route_map_kernel(RouteIdx idx, int n_sel, const int32_t* __restrict__ g_start,
                                                        const int32_t* __restrict__ g_len, int32_t* __restrict__ c_start,
                                                        int32_t* __restrict__ c_len, int32_t* __restrict__ c_src,
                                                        int32_t* __restrict__ c_seq, int32_t* __restrict__ c_n)
{
    __shared__ int len_s[kMaxRouted];
    __shared__ int start_s[kMaxRouted];
    __shared__ int part[256];
    const int tid = threadIdx.x;
    int mine = 0;
    for (int u = 0; u < 4; ++u) {
        const int i = tid * 4 + u;
        const int l = i < n_sel ? g_len[idx.seq[i]] : 0;
        if (i < kMaxRouted) len_s[i] = l;
        mine += l;
    }
    part[tid] = mine;
    __syncthreads();
    if (tid == 0) {                                   // 256 partial sums: a short serial scan
        int run = 0;
        for (int t = 0; t < 256; ++t) {
            const int v = part[t];
            part[t] = run;
            run += v;
        }
        *c_n = run;
    }
    __syncthreads();
    int run = part[tid];
    for (int u = 0; u < 4; ++u) {
        const int i = tid * 4 + u;
        if (i < n_sel) {
            start_s[i] = run;
            c_start[i] = run;
            c_len[i] = len_s[i];
            c_seq[i] = idx.seq[i];
            run += len_s[i];
        }
    }
    __syncthreads();
    for (int i = 0; i < n_sel; ++i) {
        const int src0 = g_start[idx.seq[i]], dst0 = start_s[i];
        for (int j = tid; j < len_s[i]; j += 256) c_src[dst0 + j] = src0 + j;
    }
}

// Position -> compact row of a sub-batch, for the token-level heads of routed tasks: one workgroup per sequence of
// the BATCH.  Positions of a sequence outside the sub-batch get kRowSkip (the classifier leaves them untouched),
// padded positions of a chosen sequence -1 (it writes zeros), real tokens their compact row.
__global__ __launch_bounds__(256) void route_rowof_kernel(RouteIdx idx, int n_sel, int S, const int32_t* __restrict__ row_of,
                                                          const int32_t* __restrict__ g_start, const int32_t* __restrict__ c_start,
                                                          int32_t* __restrict__ c_rowof)
{
    __shared__ int which;
    const int b = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) {
        int lo = 0, hi = n_sel - 1, found = -1;       // idx.seq is ascending
        while (lo <= hi) {
            const int mid = (lo + hi) >> 1;
            const int v = idx.seq[mid];
            if (v == b) { found = mid; break; }
            if (v < b) lo = mid + 1;
            else hi = mid - 1;
        }
        which = found;
    }
    __syncthreads();
    const int i = which;
    const int shift = i >= 0 ? c_start[i] - g_start[b] : 0;
    for (int s = tid; s < S; s += 256) {
        const size_t p = (size_t)b * S + s;
        const int r = row_of[p];
        c_rowof[p] = i < 0 ? kRowSkip : (r < 0 ? -1 : r + shift);
    }
}

__global__ __launch_bounds__(256) void route_gather_kernel(const float* __restrict__ in_f, const void* __restrict__ in_a,
                                                           float* __restrict__ out_f, void* __restrict__ out_a,
                                                           const int32_t* __restrict__ c_src, const int32_t* __restrict__ c_n,
                                                           int max_rows, int H, int act_bytes)
{
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= min(max_rows, *c_n)) return;
    const size_t src = (size_t)c_src[r];
    if (in_f && out_f)
        for (int i = lane; i < H; i += 64) out_f[(size_t)r * H + i] = in_f[src * H + i];
    if (in_a && out_a) {
        const int words = H * act_bytes / 4;
        const uint32_t* x = reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(in_a) + src * H * act_bytes);
        uint32_t* o = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(out_a) + (size_t)r * H * act_bytes);
        for (int i = lane; i < words; i += 64) o[i] = x[i];
    }
}

}  // namespace

hipError_t launch_cls_split(const SplitGroup& g, int G, int B, int H, const int32_t* seq_start, int rows_per_seq, int max_rows,
                            hipStream_t stream)
{
    if (G <= 0 || B <= 0) return hipSuccess;
    hipLaunchKernelGGL(cls_split_kernel, dim3(B, G), dim3(256), 0, stream, g, H, seq_start, rows_per_seq, max_rows);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const SplitGroup& g, int G, int B, int H, const int32_t* seq_start, int rows_per_seq, int max_rows,
                              hipStream_t stream)
{
    if (G <= 0 || B <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(B, G), dim3(256), 0, stream, g, H, seq_start, rows_per_seq, max_rows);
    return hipGetLastError();
}

hipError_t launch_gather_first_rows(const FirstRowsGroup& g, int G, int B, int H, int act_bytes, const int32_t* seq_start,
                                    int max_rows, hipStream_t stream)
{
    if (G <= 0 || B <= 0) return hipSuccess;
    if (!seq_start || (act_bytes != 2 && act_bytes != 4) || (H * act_bytes) % 4 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gather_first_rows_kernel, dim3(B, G), dim3(256), 0, stream, g, H, act_bytes, seq_start, max_rows);
    return hipGetLastError();
}

hipError_t launch_place_first_rows(const float* x, int B, int S, int H, float* out, hipStream_t stream)
{
    if (B <= 0 || S <= 0) return hipSuccess;
    const int n_pos = B * S;
    hipLaunchKernelGGL(place_first_rows_kernel, dim3((n_pos + kRowsPerBlock - 1) / kRowsPerBlock), dim3(256), 0, stream, x, n_pos, S, H,
                       out);
    return hipGetLastError();
}

hipError_t launch_token_classifier(const TokGroup& g, int G, int n_pos, int H, int w_bf16, int64_t ldo, const int32_t* row_of,
                                   const int32_t* n_rows, hipStream_t stream)
{
    if (G <= 0 || n_pos <= 0) return hipSuccess;
    if (G > kMaxGroup || !row_of || !n_rows || H < 1) return hipErrorInvalidValue;
    if (H % 256 == 0 && H <= 1280) {          // classifier rows are then 16-byte aligned for either element type
        const dim3 rgrid((n_pos + 3) / 4, G);
#define MT_TOK_ROWS(NV)                                                                                                            \
    case NV:                                                                                                                       \
        if (w_bf16) hipLaunchKernelGGL((token_classifier_rows_kernel<__bf16, NV>), rgrid, dim3(256), 0, stream, g, n_pos, ldo, row_of, n_rows); \
        else hipLaunchKernelGGL((token_classifier_rows_kernel<float, NV>), rgrid, dim3(256), 0, stream, g, n_pos, ldo, row_of, n_rows);         \
        break;
        switch (H / 256) {
            MT_TOK_ROWS(1) MT_TOK_ROWS(2) MT_TOK_ROWS(3) MT_TOK_ROWS(4) MT_TOK_ROWS(5)
        }
#undef MT_TOK_ROWS
        return hipGetLastError();
    }
    const dim3 grid((n_pos + 4 * kTokPosPerWave - 1) / (4 * kTokPosPerWave), G);
    if (w_bf16) hipLaunchKernelGGL((token_classifier_kernel<__bf16>), grid, dim3(256), 0, stream, g, n_pos, H, ldo, row_of, n_rows);
    else hipLaunchKernelGGL((token_classifier_kernel<float>), grid, dim3(256), 0, stream, g, n_pos, H, ldo, row_of, n_rows);
    return hipGetLastError();
}

// Request r's [batch_r][seq] ids and mask go to rows first[r] .. of the combined [sum batch][seq] arrays.
__global__ __launch_bounds__(256) void gather_requests_kernel(RequestPtrs rq, int seq, int32_t* __restrict__ ids_all,
                                                              int32_t* __restrict__ mask_all)
{
    const int r = blockIdx.y;
    const int32_t* __restrict__ ids = rq.ids[r];
    const int32_t* __restrict__ mask = rq.mask[r];
    const size_t base = (size_t)rq.first[r] * seq;
    const int n = (rq.first[r + 1] - rq.first[r]) * seq;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
        ids_all[base + i] = ids[i];
        mask_all[base + i] = mask[i];
    }
}

// out_r[b][c] = logits_all[first[r] + b][c] for the enabled columns c; one workgroup per (row, request)
__global__ __launch_bounds__(64) void scatter_logits_kernel(RequestPtrs rq, int n_cols, const float* __restrict__ logits_all)
{
    const int b = blockIdx.x, r = blockIdx.y;
    if (b >= rq.first[r + 1] - rq.first[r]) return;
    const float* __restrict__ src = logits_all + ((size_t)rq.first[r] + b) * n_cols;
    float* __restrict__ dst = rq.out[r] + (size_t)b * n_cols;
    for (int c = threadIdx.x; c < n_cols; c += 64)
        if ((rq.col_on[c >> 5] >> (c & 31)) & 1u) dst[c] = src[c];
}

hipError_t launch_gather_requests(const RequestPtrs& rq, int n_req, int max_batch, int seq, int32_t* ids_all, int32_t* mask_all, hipStream_t stream)
{
    if (n_req <= 0 || max_batch <= 0 || seq <= 0) return hipSuccess;
    if (n_req > kMaxRequests) return hipErrorInvalidValue;
    const int bx = (int)std::min<long>(64, ((long)max_batch * seq + 255) / 256);
    hipLaunchKernelGGL(gather_requests_kernel, dim3(bx, n_req), dim3(256), 0, stream, rq, seq, ids_all, mask_all);
    return hipGetLastError();
}

hipError_t launch_scatter_logits(const RequestPtrs& rq, int n_req, int max_batch, int n_cols, const float* logits_all, hipStream_t stream)
{
    if (n_req <= 0 || max_batch <= 0 || n_cols <= 0) return hipSuccess;
    if (n_req > kMaxRequests || n_cols > kMaxLogitCols) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scatter_logits_kernel, dim3(max_batch, n_req), dim3(64), 0, stream, rq, n_cols, logits_all);
    return hipGetLastError();
}

// bfloat16 rows -> OCP FP8 E4M3 rows at unit scale (round to nearest even, saturating): the operand copy of a layer
// input for the FP8 form of the QKV projection.  One thread converts 8 consecutive elements (16 bytes in, 8 out).
__global__ __launch_bounds__(256) void cast_bf16_to_e4m3_kernel(CastGroup g, int M, const int32_t* __restrict__ d_M, int H)
{
    if (d_M) M = min(M, *d_M);
    const size_t n8 = (size_t)M * H / 8;
    const uint4* __restrict__ src = static_cast<const uint4*>(g.src[blockIdx.y]);
    uint2* __restrict__ dst = static_cast<uint2*>(g.dst[blockIdx.y]);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const uint4 v = src[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float f[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(w[e] << 16);
            f[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
        }
        dst[i] = make_uint2(pack_e4m3(f[0], f[1], f[2], f[3]), pack_e4m3(f[4], f[5], f[6], f[7]));
    }
}

hipError_t launch_cast_bf16_to_e4m3(const CastGroup& g, int G, int M, const int32_t* d_M, int H, hipStream_t stream)
{
    if (G <= 0 || M <= 0) return hipSuccess;
    if (G > kMaxGroup || H % 8 != 0) return hipErrorInvalidValue;
    const size_t n8 = (size_t)M * H / 8;
    const int blocks = (int)std::min<size_t>((n8 + 255) / 256, 8192);
    hipLaunchKernelGGL(cast_bf16_to_e4m3_kernel, dim3(blocks, G), dim3(256), 0, stream, g, M, d_M, H);
    return hipGetLastError();
}

// One workgroup: counts the sequences whose first position is padding.
__global__ __launch_bounds__(256) void count_bad_first_tokens_kernel(const int32_t* __restrict__ mask, int B, int S, int32_t* __restrict__ count)
{
    __shared__ int part[4];
    int n = 0;
    for (int b = threadIdx.x; b < B; b += 256) n += mask[(size_t)b * S] == 0 ? 1 : 0;
    n = wave_sum_int(n);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) *count = part[0] + part[1] + part[2] + part[3];
}

hipError_t launch_count_bad_first_tokens(const int32_t* mask, int B, int S, int32_t* count, hipStream_t stream)
{
    if (B <= 0 || S <= 0 || !mask || !count) return hipErrorInvalidValue;
    hipLaunchKernelGGL(count_bad_first_tokens_kernel, dim3(1), dim3(256), 0, stream, mask, B, S, count);
    return hipGetLastError();
}

hipError_t launch_build_row_map(const int32_t* mask, int B, int S, const RowMap& map, hipStream_t stream)
{
    if (B <= 0 || S <= 0) return hipSuccess;
    hipLaunchKernelGGL(row_rank_kernel, dim3(B), dim3(256), 0, stream, mask, S, map.row_of, map.seq_len);
    hipLaunchKernelGGL(row_place_kernel, dim3(B), dim3(256), 0, stream, B, S, map.row_of, map.seq_len, map.seq_start, map.src,
                       map.n_rows);
    return hipGetLastError();
}

hipError_t launch_unpack_rows(const float* x, const int32_t* row_of, int n_pos, int H, float* out, hipStream_t stream)
{
    if (n_pos <= 0) return hipSuccess;
    hipLaunchKernelGGL(unpack_rows_kernel, dim3((n_pos + kRowsPerBlock - 1) / kRowsPerBlock), dim3(256), 0, stream, x, row_of,
                       n_pos, H, out);
    return hipGetLastError();
}

hipError_t launch_classifier(const ClsGroup& g, int G, int B, int H, int maxC, int w_bf16, int64_t ldo, const int32_t* out_row,
                             hipStream_t stream)
{
    if (G <= 0 || B <= 0 || maxC <= 0) return hipSuccess;
    const dim3 grid(B, G, (maxC + 3) / 4);
    if (w_bf16) hipLaunchKernelGGL((classifier_kernel<__bf16>), grid, dim3(256), 0, stream, g, B, H, ldo, out_row);
    else hipLaunchKernelGGL((classifier_kernel<float>), grid, dim3(256), 0, stream, g, B, H, ldo, out_row);
    return hipGetLastError();
}

hipError_t launch_route_map(const RouteIdx& idx, int n_sel, const int32_t* g_start, const int32_t* g_len, int32_t* c_start,
                            int32_t* c_len, int32_t* c_src, int32_t* c_seq, int32_t* c_n, hipStream_t stream)
{
    if (n_sel <= 0) return hipSuccess;
    if (n_sel > kMaxRouted || !g_start || !g_len || !c_start || !c_len || !c_src || !c_seq || !c_n) return hipErrorInvalidValue;
    hipLaunchKernelGGL(route_map_kernel, dim3(1), dim3(256), 0, stream, idx, n_sel, g_start, g_len, c_start, c_len, c_src, c_seq, c_n);
    return hipGetLastError();
}

hipError_t launch_route_rowof(const RouteIdx& idx, int n_sel, int B, int S, const int32_t* row_of, const int32_t* g_start,
                              const int32_t* c_start, int32_t* c_rowof, hipStream_t stream)
{
    if (B <= 0 || S <= 0) return hipSuccess;
    if (n_sel < 0 || n_sel > kMaxRouted || !row_of || !g_start || !c_start || !c_rowof) return hipErrorInvalidValue;
    hipLaunchKernelGGL(route_rowof_kernel, dim3(B), dim3(256), 0, stream, idx, n_sel, S, row_of, g_start, c_start, c_rowof);
    return hipGetLastError();
}

hipError_t launch_route_gather(const float* in_f, const void* in_a, float* out_f, void* out_a, const int32_t* c_src, const int32_t* c_n,
                               int max_rows, int H, int act_bytes, hipStream_t stream)
{
    if (max_rows <= 0) return hipSuccess;
    if (!c_src || !c_n || (act_bytes != 2 && act_bytes != 4) || (H * act_bytes) % 4 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(route_gather_kernel, dim3((max_rows + kRowsPerBlock - 1) / kRowsPerBlock), dim3(256), 0, stream, in_f, in_a, out_f,
                       out_a, c_src, c_n, max_rows, H, act_bytes);
    return hipGetLastError();
}

hipError_t launch_layernorm(const LnGroup& g, int G, int M, const int32_t* d_M, int H, float eps, int n_parts, int64_t part_stride,
                            hipStream_t stream, int low_fmt)
{
    if (G <= 0 || M <= 0) return hipSuccess;
    if (low_fmt != 0 && low_fmt != 1) return hipErrorInvalidValue;
    dim3 grid((M + kRowsPerBlock - 1) / kRowsPerBlock, G), block(256);
    if (H == 768) hipLaunchKernelGGL((layernorm_fast<3>), grid, block, 0, stream, g, M, d_M, H, eps, n_parts, part_stride, low_fmt);
    else if (H == 1024) hipLaunchKernelGGL((layernorm_fast<4>), grid, block, 0, stream, g, M, d_M, H, eps, n_parts, part_stride, low_fmt);
    else if (H == 512) hipLaunchKernelGGL((layernorm_fast<2>), grid, block, 0, stream, g, M, d_M, H, eps, n_parts, part_stride, low_fmt);
    else if (H == 256) hipLaunchKernelGGL((layernorm_fast<1>), grid, block, 0, stream, g, M, d_M, H, eps, n_parts, part_stride, low_fmt);
    else hipLaunchKernelGGL(layernorm_any, grid, block, 0, stream, g, M, d_M, H, eps, n_parts, part_stride, low_fmt);
    return hipGetLastError();
}

hipError_t launch_embed_ln(const int32_t* ids, const int32_t* type_ids, int type_vocab, const int32_t* src, const int32_t* d_M, int B, int S, int H, int vocab, const void* word, const void* pos,
                           const void* type, int emb_bf16, const float* gamma, const float* beta, float eps,
                           float* out_f32, bf16_t* out_bf16, hipStream_t stream)
{
    if (B * S <= 0) return hipSuccess;
    __bf16* ob = reinterpret_cast<__bf16*>(out_bf16);
    if (emb_bf16)
        return embed_dispatch<__bf16>(ids, type_ids, type_vocab, src, d_M, B, S, H, vocab, (const __bf16*)word, (const __bf16*)pos, (const __bf16*)type,
                                      gamma, beta, eps, out_f32, ob, stream);
    return embed_dispatch<float>(ids, type_ids, type_vocab, src, d_M, B, S, H, vocab, (const float*)word, (const float*)pos, (const float*)type,
                                 gamma, beta, eps, out_f32, ob, stream);
}

}  // namespace mt
