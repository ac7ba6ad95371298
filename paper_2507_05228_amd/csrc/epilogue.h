// Scalar pieces of the shard-GEMM epilogue, shared by the fp32 and the bf16 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/cascade.h"

__device__ __forceinline__ float gelu_erf_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

__device__ __forceinline__ float gelu_tanh_f(float x) {
    float t = 0.79788456080286536f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(t));
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

__device__ __forceinline__ float apply_act(float v, int flags) {
    if (flags & CASCADE_EPI_GELU_ERF) return gelu_erf_f(v);
    if (flags & CASCADE_EPI_GELU_TANH) return gelu_tanh_f(v);
    return v;
}

// The same activations for results that are rounded to bf16 (2^-9 relative): the error function by the rational
// approximation 7.1.26 of Abramowitz and Stegun's handbook (absolute error below 1.5e-7) and tanh through one
// exponential, both on the hardware's exp2 and reciprocal: a fifth of the instructions of the library routines,
// which the epilogue of a short-reduction GEMM is otherwise dominated by.
__device__ __forceinline__ float erf_fast(float x) {
    const float z = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * z * z);
    return copysignf(1.0f - poly * t * e, x);
}
__device__ __forceinline__ float gelu_erf_fast(float x) { return 0.5f * x * (1.0f + erf_fast(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_tanh_fast(float x) {
    const float t = 0.79788456080286536f * (x + 0.044715f * x * x * x);
    // tanh t = 1 - 2 / (1 + e^(2t)); e^(2t) = inf gives 1, 0 gives -1
    const float th = 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * t));
    return 0.5f * x * (1.0f + th);
}
__device__ __forceinline__ float apply_act_bf16(float v, int flags) {
    if (flags & CASCADE_EPI_GELU_ERF) return gelu_erf_fast(v);
    if (flags & CASCADE_EPI_GELU_TANH) return gelu_tanh_fast(v);
    return v;
}

// Weight rows are stacked in up to three segments along the output axis (q | k | v).
struct WeightSegs {
    const void *w[3];
    const void *bias[3];
    int32_t end[3];
};

template <typename T>
__device__ __forceinline__ const T *weight_row(const WeightSegs &s, int n, int64_t K) {
    if (n < s.end[0]) return (const T *)s.w[0] + (int64_t)n * K;
    if (n < s.end[1]) return (const T *)s.w[1] + (int64_t)(n - s.end[0]) * K;
    return (const T *)s.w[2] + (int64_t)(n - s.end[1]) * K;
}

template <typename T>
__device__ __forceinline__ float bias_at(const WeightSegs &s, int n) {
    const T *b;
    int off;
    if (n < s.end[0]) { b = (const T *)s.bias[0]; off = n; }
    else if (n < s.end[1]) { b = (const T *)s.bias[1]; off = n - s.end[0]; }
    else { b = (const T *)s.bias[2]; off = n - s.end[1]; }
    return b ? (float)b[off] : 0.f;
}
