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
// The erf form for bf16 epilogues.  GELU(x) = x * Phi(x) and Phi(x) = 1 / (1 + exp(-z(x))) with z = ln(Phi(x) / Phi(-x)),
// an odd function of x; z is replaced by the odd polynomial x * (c0 + c1 x^2 + c2 x^4) whose coefficients minimise the
// largest absolute error of x * Phi(x) on [-9, 9] (fitted against erf in float64: 2.6e-5, reached near x = -0.56; the
// published tanh form, the same shape with two coefficients chosen differently, is off by 4.7e-4).  That is a
// twentieth of the bf16 rounding step of a typical activation (0.3 .. 1) and is what every bf16 kernel stores;
// the float32 validation mode uses erff.  6 multiply-adds, one exp2, one reciprocal per element.
__device__ __forceinline__ float gelu_erf_fast(float x)
{
    constexpr float kLog2e = 1.4426950408889634f;
    const float xc = __builtin_amdgcn_fmed3f(x, -9.0f, 9.0f);  // the fit's range; beyond it Phi is 0 or 1 to float32 anyway
    const float x2 = xc * xc;
    float p = fmaf(x2, -7.03037878e-04f * kLog2e, 7.40113199e-02f * kLog2e);
    p = fmaf(x2, p, 1.59501574e+00f * kLog2e);
    const float e = __builtin_amdgcn_exp2f(-xc * p);          // exp(-z), between 2^-39 and 2^39
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ inline float gelu_tanh(float x)
{
    const float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
}

// four float32 -> four OCP FP8 E4M3 bytes in one dword (round to nearest even, saturating at +-448)
__device__ __forceinline__ uint32_t pack_e4m3(float a, float b, float c, float d)
{
    a = __builtin_amdgcn_fmed3f(a, -448.f, 448.f);
    b = __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
    c = __builtin_amdgcn_fmed3f(c, -448.f, 448.f);
    d = __builtin_amdgcn_fmed3f(d, -448.f, 448.f);
    int v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
    return (uint32_t)v;
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
