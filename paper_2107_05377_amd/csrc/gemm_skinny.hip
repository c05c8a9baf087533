// bfloat16 contraction for FEW rows (the first-token-only last layer of every branch, the pooler, and
// small-batch serving):  C_g[M,N] = epi(A_g[M,K] * W_g[N,K]^T) with M of a few dozen rows.
// Such a problem is bound by streaming the weights, not by the matrix cores, so the kernel is laid out for
// memory parallelism instead of operand reuse:
//   - a workgroup owns a 32-row x 32-column output block; its 4 wavefronts each take a quarter of the
//     K range and multiply straight from global memory (every lane fetches its own 16-byte MFMA
//     fragments of A and W, 12 K-steps in flight: a quarter of K = 768 in one round trip), so every weight byte is fetched exactly once per
//     32-row block and there are N/32 x G (x splits) workgroups to spread the stream over the chip;
//   - the four partial 32x32 tiles meet in LDS, are added in a fixed order, and all 256 threads apply
//     bias / activation / residual to 4 consecutive columns each and store whole row segments.
// K may additionally be split over workgroups (float32 partial outputs, summed by the next LayerNorm).
#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int SK_BM = 32, SK_BN = 32;
constexpr int SK_UNROLL = 12;          // K steps (of 16) in flight per wavefront
constexpr int SK_LDP = SK_BN + 4;     // padded row of the float32 partial tile in LDS

__device__ __forceinline__ float skinny_act(float v, int act)
{
    switch (act) {
        case ACT_GELU_ERF: return gelu_erf_fast(v);
        case ACT_GELU_TANH: return gelu_tanh(v);
        case ACT_TANH: return tanhf(v);
        default: return v;
    }
}

template <bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_skinny_bf16_kernel(GemmGroup g, GemmShape s)
{
    __shared__ __attribute__((aligned(16))) float part[4][SK_BM][SK_LDP];
    const int nsub = s.n_sub > 1 ? s.n_sub : 1;
    const int sub = blockIdx.z % nsub, gz = blockIdx.z / nsub;
    const int grp = gz / s.splits, split = gz - grp * s.splits;
    int M = s.d_M ? min(s.M, *s.d_M) : s.M;
    size_t row_base = 0;                                   // ragged batch: this sub-problem's rows of A and C
    if (s.d_sub_rows) {
        M = min(s.M, s.d_sub_rows[sub]);
        row_base = (size_t)s.d_sub_row0[sub];
    }
    const int m0 = blockIdx.y * SK_BM;
    if (m0 >= M) return;
    const int n0 = blockIdx.x * SK_BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;

    // this wavefront's K range: a quarter of this workgroup's range
    const int k_len = s.K / s.splits / 4;
    const int k_begin = split * (s.K / s.splits) + wave * k_len;
    const __bf16* __restrict__ a_row =
        static_cast<const __bf16*>(g.A[grp]) + (size_t)sub * s.sub_a + (row_base + min(m0 + l32, M - 1)) * s.lda + k_begin + half * 8;
    const __bf16* __restrict__ w_row =
        static_cast<const __bf16*>(g.W[grp]) + (size_t)sub * s.sub_w + (size_t)min(n0 + l32, s.N - 1) * (s.ldw ? s.ldw : s.K) + k_begin + half * 8;

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    const int steps = k_len / 16;
    int st = 0;
    for (; st + SK_UNROLL <= steps; st += SK_UNROLL) {
        bf16x8 af[SK_UNROLL], wf[SK_UNROLL];
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u) {
            af[u] = *reinterpret_cast<const bf16x8*>(a_row + (st + u) * 16);
            wf[u] = *reinterpret_cast<const bf16x8*>(w_row + (st + u) * 16);
        }
        // nothing moves across this point: without it the scheduler sinks the loads between the matrix instructions and
        // keeps only five of them in flight (seen in the kernel's own assembly), i.e. a third of the bytes per round trip
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], af[u], acc, 0, 0, 0);
    }
    if (st < steps) {      // the last, shorter batch (nb is uniform over the workgroup): again one round trip
        const int nb = steps - st;
        bf16x8 af[SK_UNROLL], wf[SK_UNROLL];
#pragma unroll
        for (int u = 0; u < SK_UNROLL - 1; ++u) {
            if (u < nb) {
                af[u] = *reinterpret_cast<const bf16x8*>(a_row + (st + u) * 16);
                wf[u] = *reinterpret_cast<const bf16x8*>(w_row + (st + u) * 16);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < SK_UNROLL - 1; ++u)
            if (u < nb) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], af[u], acc, 0, 0, 0);
    }
    // lane holds row m = l32, columns n = 8q + 4*half + {0..3}
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&part[wave][l32][q * 8 + half * 4]) =
            make_float4(acc[q * 4 + 0], acc[q * 4 + 1], acc[q * 4 + 2], acc[q * 4 + 3]);
    __syncthreads();

    const int r = tid >> 3, c4 = (tid & 7) * 4;
    const int m = m0 + r, n = n0 + c4;
    if (m >= M || n >= s.N) return;            // N % 4 == 0: a thread's 4 columns are all in or all out
    float4 v = *reinterpret_cast<const float4*>(&part[0][r][c4]);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const float4 t = *reinterpret_cast<const float4*>(&part[w][r][c4]);
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
    if (g.bias[grp]) {
        const float4 b = *reinterpret_cast<const float4*>(g.bias[grp] + (size_t)sub * s.sub_bias + n);
        v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
    }
    v.x = skinny_act(v.x, s.act);
    v.y = skinny_act(v.y, s.act);
    v.z = skinny_act(v.z, s.act);
    v.w = skinny_act(v.w, s.act);
    if constexpr (OUT_F32) {
        if (g.residual[grp]) {
            const float4 t = *reinterpret_cast<const float4*>(g.residual[grp] + (size_t)m * s.ldr + n);
            v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
        }
        float* C = static_cast<float*>(g.C[grp]) + (size_t)split * s.split_stride + (size_t)sub * s.sub_c;
        *reinterpret_cast<float4*>(C + (row_base + m) * s.ldc + n) = v;
    } else {
        bf16x4 o = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
        *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(g.C[grp]) + (size_t)sub * s.sub_c + (row_base + m) * s.ldc + n) = o;
    }
}

}  // namespace

bool gemm_skinny_applicable(const GemmShape& s) { return s.M <= 256; }

hipError_t launch_gemm_skinny_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream)
{
    if (s.G <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
    if (s.splits < 1 || (s.splits > 1 && (!s.out_f32 || s.act != ACT_NONE || g.bias[0] || g.residual[0]))) return hipErrorInvalidValue;
    if (s.K % (64 * s.splits) != 0 || s.N % 4 != 0 || s.lda % 8 != 0 || s.ldw % 8 != 0 || (s.ldw && s.ldw < s.K) || s.ldc % 4 != 0 || s.ldr % 4 != 0 || s.G > kMaxGroup ||
        (!s.out_f32 && g.residual[0] != nullptr))
        return hipErrorInvalidValue;
    const int nsub = s.n_sub > 1 ? s.n_sub : 1;
    if ((long)s.G * s.splits * nsub > 65535) return hipErrorInvalidValue;
    if (nsub > 1 && (g.residual[0] != nullptr || s.d_M != nullptr || s.sub_a % 8 != 0 || s.sub_w % 8 != 0 || s.sub_c % 4 != 0 ||
                     s.sub_bias % 4 != 0))
        return hipErrorInvalidValue;
    if ((s.d_sub_rows != nullptr) != (s.d_sub_row0 != nullptr) || (s.d_sub_rows && (s.d_M != nullptr || g.residual[0] != nullptr)))
        return hipErrorInvalidValue;
    dim3 grid((s.N + SK_BN - 1) / SK_BN, (s.M + SK_BM - 1) / SK_BM, s.G * s.splits * nsub), block(256);
    if (s.out_f32) hipLaunchKernelGGL((gemm_skinny_bf16_kernel<true>), grid, block, 0, stream, g, s);
    else hipLaunchKernelGGL((gemm_skinny_bf16_kernel<false>), grid, block, 0, stream, g, s);
    return hipGetLastError();
}

}  // namespace mt
