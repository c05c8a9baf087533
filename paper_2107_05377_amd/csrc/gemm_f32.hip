// float32 contraction on the vector ALUs: C_g[M,N_g] = epi(A_g[M,K] * W_g[N_g,K]^T) for a group of problems.
// Used by the float32 validation mode for every linear layer, and in both modes for the pooler and
// classifier (their inputs stay float32 so that the logits do not inherit a bfloat16 rounding).
// 64x64 output tile per 256-thread block, 4x4 outputs per thread, K staged through LDS in slices of 16.
// Any M, N, K, lda: loads outside the problem are zero-filled, stores are bounds-checked.
#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename TW>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmGroup g, GemmShape s)
{
    __shared__ float As[TK][TM + 4];
    __shared__ float Ws[TK][TN + 4];
    const int grp = blockIdx.z;
    const int N = g.N[grp];
    const int M = s.d_M ? min(s.M, *s.d_M) : s.M;      // rows actually present; the grid covers the bound s.M
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    if (n0 >= N || m0 >= M) return;
    const float* A = static_cast<const float*>(g.A[grp]);
    const TW* W = static_cast<const TW*>(g.W[grp]);
    const size_t ldw = s.ldw ? s.ldw : s.K;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int lr = threadIdx.x >> 2;          // 0..63: tile row loaded by this thread
    const int lk = (threadIdx.x & 3) * 4;     // 0,4,8,12: first of 4 k's
    float acc[4][4] = {};
    for (int k0 = 0; k0 < s.K; k0 += TK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + lk + j;
            const int am = m0 + lr, wn = n0 + lr;
            As[lk + j][lr] = (am < M && k < s.K) ? A[(size_t)am * s.lda + k] : 0.f;
            Ws[lk + j][lr] = (wn < N && k < s.K) ? (float)W[(size_t)wn * ldw + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; w[i] = Ws[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* C = static_cast<float*>(g.C[grp]);
    const float* bias = g.bias[grp];
    const float* res = g.residual[grp];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j] + (bias ? bias[n] : 0.f);
            v = apply_act(v, s.act);
            if (res) v += res[(size_t)m * s.ldr + n];
            C[(size_t)m * s.ldc + n] = v;
        }
    }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmGroup& g, const GemmShape& s, int w_bf16, hipStream_t stream)
{
    if (s.G <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
    dim3 grid((s.N + TN - 1) / TN, (s.M + TM - 1) / TM, s.G), block(256);
    if (w_bf16) hipLaunchKernelGGL((gemm_f32_kernel<__bf16>), grid, block, 0, stream, g, s);
    else hipLaunchKernelGGL((gemm_f32_kernel<float>), grid, block, 0, stream, g, s);
    return hipGetLastError();
}

}  // namespace mt
