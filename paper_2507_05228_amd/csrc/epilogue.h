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
