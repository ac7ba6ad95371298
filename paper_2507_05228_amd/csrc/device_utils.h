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

// Wavefront reductions; every lane gets the result.  Inside a 16-lane row the partner's value comes
// through a data-parallel-primitive move (lanes ^1, ^2 by quad permutes, then the half-row and row
// mirrors: for a symmetric reduction a reversal is as good as a swap) and costs no LDS traffic; the
// four rows are combined with two cross-row shuffles.
template <int CTRL>
__device__ __forceinline__ float dpp_row_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_row_move<0xB1>(v));      // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_row_move<0x4E>(v));      // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_row_move<0x141>(v));     // row_half_mirror
    v = fmaxf(v, dpp_row_move<0x140>(v));     // row_mirror
    v = fmaxf(v, __shfl_xor(v, 16, WAVE));
    return fmaxf(v, __shfl_xor(v, 32, WAVE));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_row_move<0xB1>(v);
    v += dpp_row_move<0x4E>(v);
    v += dpp_row_move<0x141>(v);
    v += dpp_row_move<0x140>(v);
    v += __shfl_xor(v, 16, WAVE);
    return v + __shfl_xor(v, 32, WAVE);
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
    if (r < seq_len) return map[r];                        // the first (or only) sequence: no division
    int32_t b = r / seq_len;
    return (int64_t)b * seq_len + map[r - b * seq_len];
}
// The same for a row known to lie in or shortly behind sequence b_hint (the rows of a tile whose first row lies in
// that sequence): a subtraction and a compare instead of an integer division by a run-time divisor, which costs
// ~40 instructions per row and was most of the time of an epilogue that looks up 8 to 32 rows per lane.
__device__ __forceinline__ int64_t map_row_near(const int32_t *map, int32_t seq_len, int32_t r, int32_t b_hint) {
    if (!map) return r;
    const int32_t off = r - b_hint * seq_len;
    if ((uint32_t)off < (uint32_t)seq_len) return (int64_t)b_hint * seq_len + map[off];
    return map_row(map, seq_len, r);
}
// N rows of one tile at once (a negative r[i] passes through).  map_row_near has three ways out, so a sequence of
// calls compiles to a branch, a load and a wait per row, one memory round trip each (16 rows: most of an epilogue
// that runs once); here the lookups of a wavefront whose rows all lie in sequence b_hint go out back to back.
template <int N>
__device__ __forceinline__ void map_rows_near(const int32_t *map, int32_t seq_len, const int32_t (&r)[N], int32_t b_hint,
                                              int32_t (&out)[N]) {
    if (!map) {
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = r[i];
        return;
    }
    const int32_t base = b_hint * seq_len;
    bool near = true;
#pragma unroll
    for (int i = 0; i < N; ++i) near &= r[i] < 0 || (uint32_t)(r[i] - base) < (uint32_t)seq_len;
    if (__all(near)) {
        int32_t v[N];
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = map[r[i] < 0 ? 0 : r[i] - base];
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = r[i] < 0 ? r[i] : base + v[i];
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = r[i] < 0 ? r[i] : (int32_t)map_row(map, seq_len, r[i]);
    }
}
