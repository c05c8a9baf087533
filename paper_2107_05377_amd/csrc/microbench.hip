// Matrix-core rate of the chip as it runs here, for judging the contraction kernels against more than the
// data-sheet figure: every SIMD issues back-to-back, independent v_mfma_f32_32x32x16_bf16 on registers only
// (no LDS, no memory), two wavefronts per SIMD.  The result moves with the clock the power management
// grants under full matrix load, which is below the boost clock the data-sheet peak assumes, and that clock
// depends on how many operand bits toggle: the operands are pseudo-random bfloat16 values in +-[0.5, 1), like
// activations and weights (with small constant integers the same loop runs 25-30 % faster).
#include "kernels.h"
#include "device_util.h"

namespace mt {

namespace {

constexpr int MB_ACC = 8;          // independent accumulators per wavefront
constexpr int MB_THREADS = 512;    // 8 wavefronts: 2 per SIMD

__global__ __launch_bounds__(MB_THREADS) void mfma_rate_kernel(float* __restrict__ out, int iters)
{
    f32x16 acc[MB_ACC];
#pragma unroll
    for (int i = 0; i < MB_ACC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 a[4], b[2];
    auto value = [](unsigned key) {            // a bfloat16 with random sign and mantissa, exponent of 0.5
        unsigned h = key * 2654435761u;
        h ^= h >> 13;
        h *= 0x5bd1e995u;
        h ^= h >> 15;
        const unsigned bits = ((h & 0x807fu) | 0x3f00u) << 16;
        return (__bf16)__uint_as_float(bits);
    };
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[i][e] = value((blockIdx.x * MB_THREADS + threadIdx.x) * 64u + i * 8 + e);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) b[i][e] = value((blockIdx.x * MB_THREADS + threadIdx.x) * 64u + 32 + i * 8 + e);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < MB_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[i & 1], a[i >> 1], acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MB_ACC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[(size_t)blockIdx.x * MB_THREADS + threadIdx.x] = s;     // keeps the loop alive
}

}  // namespace

hipError_t run_mfma_rate(int iters, int n_cu, float* d_out, hipStream_t stream, float* tflops)
{
    hipEvent_t e0, e1;
    hipError_t err = hipEventCreate(&e0);
    if (err != hipSuccess) return err;
    err = hipEventCreate(&e1);
    if (err != hipSuccess) { (void)hipEventDestroy(e0); return err; }
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_cu), dim3(MB_THREADS), 0, stream, d_out, iters / 4 + 1);   // warm-up, clocks settle
    (void)hipEventRecord(e0, stream);
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_cu), dim3(MB_THREADS), 0, stream, d_out, iters);
    (void)hipEventRecord(e1, stream);
    err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    if (err == hipSuccess) err = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess) return err;
    const double flops = 2.0 * 32 * 32 * 16 * (double)MB_ACC * iters * (MB_THREADS / 64) * n_cu;
    *tflops = (float)(flops / (ms * 1e-3) / 1e12);
    return hipSuccess;
}

int mfma_rate_out_floats(int n_cu) { return n_cu * MB_THREADS; }

}  // namespace mt
