// Shared host/device helpers of libhyb (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/hyb.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define HYB_WAVE 64

// ---- error reporting -----------------------------------------------------------------------
int hyb_set_error(int code, const char* fmt, ...);

#define HYB_REQUIRE(cond, code, ...)                         \
    do {                                                     \
        if (!(cond)) return hyb_set_error((code), __VA_ARGS__); \
    } while (0)

#define HYB_CHECK_PTR(p) HYB_REQUIRE((p) != nullptr, HYB_ERR_NULL, "%s: argument '%s' is NULL", __func__, #p)
#define HYB_CHECK_ALIGN(p) \
    HYB_REQUIRE((((uintptr_t)(p)) & 15u) == 0, HYB_ERR_ALIGN, "%s: argument '%s' is not 16-byte aligned", __func__, #p)
#define HYB_CHECK_DTYPE(d) \
    HYB_REQUIRE((d) == HYB_F32 || (d) == HYB_BF16, HYB_ERR_DTYPE, "%s: argument '%s' is not a valid dtype", __func__, #d)

int hyb_check_launch(const char* what);

// ---- optional per-launch timing (hyb_trace_*) ----------------------------------------------
// A scope object brackets one kernel launch with two events on the launch stream when tracing
// is on; `work` is the algorithmic work of the launch (flops or bytes, `unit` says which).
struct HybTraceScope {
    int slot;
    hipStream_t st;
    HybTraceScope(const char* kernel, const char* unit, double work, hipStream_t stream);
    ~HybTraceScope();
};

static inline size_t hyb_dtype_size(hyb_dtype d) { return d == HYB_BF16 ? 2 : 4; }
static inline size_t hyb_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- device helpers ------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short u) { return __uint_as_float(((unsigned int)u) << 16); }

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sigmoid-shaped activations use the hardware reciprocal (1 ulp) instead of an IEEE division: the
// correctly rounded quotient costs about ten extra instructions per element in the GEMM epilogues.
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float gelu_tanh_f(float z) {
    // 0.5 z (1 + tanh(u)) = z * sigmoid(2u) = z / (1 + 2^(-2 u log2(e))), u = sqrt(2/pi) (z + 0.044715 z^3); the constants
    // are folded into the cubic, so that an element costs seven instructions: -2 u log2(e) = z (k1 + k3 z^2)
    constexpr float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    constexpr float k3 = k1 * 0.044715f;
    const float arg = z * fmaf(z * z, k3, k1);
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(arg));
}
// Exact-erf GELU with erf from the rational approximation 7.1.26 of Abramowitz & Stegun,
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0 (absolute error < 1.5e-7, far inside
// the fp32 tolerance of the workloads), a dozen instructions instead of the library routine's branches.
__device__ __forceinline__ float gelu_erf_f(float z) {
    const float x = fabsf(z) * 0.7071067811865476f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float erf_abs = 1.0f - poly * t * __expf(-x * x);
    return 0.5f * z * (1.0f + copysignf(erf_abs, z));
}
