// Device-side helpers for gfx950: bf16 vectors, wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define WAVE 64

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return (float)x; }
__device__ __forceinline__ bf16_t f32_to_bf16(float x) { return (bf16_t)x; }   // v_cvt_pk_bf16_f32: round to nearest even

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return (float)*p; }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = (bf16_t)v; }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// Sum over a 256-thread block; scratch holds >= 4 floats.  Every thread gets the result.
__device__ __forceinline__ float block_sum_256(float v, float *scratch) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

__device__ __forceinline__ int64_t map_row(const int32_t *map, int32_t seq_len, int32_t r) {
    if (!map) return r;
    int32_t b = r / seq_len;
    return (int64_t)b * seq_len + map[r - b * seq_len];
}
