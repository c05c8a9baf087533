// Small device helpers shared by the gfx950 kernels: vector types, wavefront reductions, activations.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

namespace mt {

// Host: raise a kernel's dynamic-LDS limit once per device (the attribute belongs to the function ON a device).
// `done` is the call site's bit set of devices already served; concurrent first calls both set the same value.
inline hipError_t ensure_dynamic_lds(const void* fn, int bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Sum / max over the 64 lanes of a wavefront; every lane receives the result.
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ inline int wave_sum_int(int v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// GELU(x) = x * Phi(x).  Exact form through erff; tanh form as the published approximation.
__device__ inline float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
// The erf form for bf16 epilogues: erf through the Abramowitz-Stegun 7.1.26 rational (|error| <= 1.5e-7 before
// rounding), far below the bf16 rounding of the stored result.  The one fast form every bf16 kernel uses.
__device__ __forceinline__ float gelu_erf_fast(float x)
{
    const float ax = fabsf(x);
    const float y = ax * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, y, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(-y * y * 1.4426950408889634f);
    const float erf_abs = fmaf(-p, e, 1.0f);          // erf(|x|/sqrt2)
    return 0.5f * fmaf(ax, erf_abs, x);               // 0.5*(x + |x| erf(|x|/sqrt2)) = x*Phi(x)
}
__device__ inline float gelu_tanh(float x)
{
    const float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
}

__device__ inline float apply_act(float v, int act)
{
    switch (act) {
        case 1: return gelu_erf(v);
        case 2: return gelu_tanh(v);
        case 3: return tanhf(v);
        default: return v;
    }
}

}  // namespace mt
