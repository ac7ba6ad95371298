// HBM-bound per-token kernels: normalisation with row gather (the optional normalisation step of the
// Pre-Pass subsection), rotary embedding at original token positions
// (the rotary step of Algorithm 2).  The gather into packed order is the row map of the norm's read; the
// scatter back is the row map of the last shard GEMM's store.
#include <climits>
#include <cmath>
#include "common.h"
#include "device_utils.h"

// ---------------------------------------------------------------------------- rotary angles
// cos and sin of position * theta^(-2i/d), i < d/2.  The angle is carried in revolutions: rev = theta^(-2i/d) /
// (2 pi) in double precision, split into two floats, and position * rev is formed with a compensated product, so
// the fractional part (all that sine and cosine need) stays accurate to ~1e-7 revolutions however large the
// position (below 2^24); sine and cosine are then single hardware instructions.
struct RopeRev { float hi, lo; };
__device__ __forceinline__ RopeRev rope_rev(float theta, int i, int head_dim) {
    const double rev = exp2(-2.0 * i / head_dim * log2((double)theta)) / 6.283185307179586476925;
    RopeRev r;
    r.hi = (float)rev;
    r.lo = (float)(rev - (double)r.hi);
    return r;
}
__device__ __forceinline__ void rope_cos_sin(float pos, float c_hi, float c_lo, float &cs, float &sn) {
    const float r_hi = pos * c_hi;
    const float r_err = fmaf(pos, c_hi, -r_hi) + pos * c_lo;      // pos * (hi + lo) = r_hi + r_err
    const float rev = (r_hi - floorf(r_hi)) + r_err;
    sn = __builtin_amdgcn_sinf(rev);
    cs = __builtin_amdgcn_cosf(rev);
}
// By-product of the pre-pass norm: the workgroup of row r writes that row's cos | sin table (the shard GEMM
// that follows rotates q and k with it in its epilogue).
struct RopeTableOut {
    float *table;
    const int32_t *pos;
    int32_t seq_len, head_dim;
    float theta;
};
// Second by-product: a few words cleared by the first workgroup (the flags of the split-reduction shard GEMMs that
// follow in the stream; a fill of its own would cost a launch, and a memset cannot be captured in a graph).
struct ZeroWords {
    uint32_t *words;
    int32_t n;
};
__device__ __forceinline__ void clear_words(const ZeroWords &z) {
    if (z.words && blockIdx.x == 0)
        for (int i = threadIdx.x; i < z.n; i += blockDim.x) z.words[i] = 0u;
}
__device__ __forceinline__ void write_rope_row(const RopeTableOut &t, int r) {
    const int half = t.head_dim >> 1;
    const float pos = (float)t.pos[r % t.seq_len];
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        const RopeRev c = rope_rev(t.theta, i, t.head_dim);
        float cs, sn;
        rope_cos_sin(pos, c.hi, c.lo, cs, sn);
        t.table[(int64_t)r * t.head_dim + i] = cs;
        t.table[(int64_t)r * t.head_dim + half + i] = sn;
    }
}

// ---------------------------------------------------------------------------- norm
// One 256-thread block per row; the row is staged in LDS as fp32 (D * 4 bytes).
template <typename T>
__global__ __launch_bounds__(256) void norm_kernel(const T *__restrict__ x, const T *__restrict__ gain,
                                                   const T *__restrict__ bias, T *__restrict__ y, int D, int kind,
                                                   float eps, const int32_t *xmap, const int32_t *ymap, int seq_len,
                                                   RopeTableOut rope, ZeroWords zero) {
    extern __shared__ float row[];
    __shared__ float red[4];
    const int r = blockIdx.x;
    clear_words(zero);
    if (rope.table) write_rope_row(rope, r);
    const T *xr = x + map_row(xmap, seq_len, r) * (int64_t)D;
    float s = 0.f;
    for (int i = threadIdx.x; i < D; i += 256) {
        float v = Elem<T>::load(xr + i);
        row[i] = v;
        s += v;
    }
    float mu = 0.f;
    if (kind == CASCADE_NORM_LAYERNORM) mu = block_sum_256(s, red) / D;
    float q = 0.f;
    for (int i = threadIdx.x; i < D; i += 256) {
        float c = row[i] - mu;
        q += c * c;
    }
    float var = block_sum_256(q, red) / D;
    float rstd = 1.0f / sqrtf(var + eps);
    T *yr = y + map_row(ymap, seq_len, r) * (int64_t)D;
    for (int i = threadIdx.x; i < D; i += 256) {
        float v = (row[i] - mu) * rstd * Elem<T>::load(gain + i);
        if (bias) v += Elem<T>::load(bias + i);
        Elem<T>::store(yr + i, v);
    }
}

// Vector variant: the row lives in registers (CH 16-byte pieces per thread), two passes over them.
// Requires D % VEC == 0 and D <= 256 * CH * VEC, VEC = 16 bytes / sizeof(T).
template <typename T, int CH>
__global__ __launch_bounds__(256) void norm_vec_kernel(const T *__restrict__ x, const T *__restrict__ gain,
                                                       const T *__restrict__ bias, T *__restrict__ y, int D, int kind,
                                                       float eps, const int32_t *xmap, const int32_t *ymap, int seq_len,
                                                       RopeTableOut rope, ZeroWords zero) {
    constexpr int VEC = 16 / sizeof(T);
    typedef T vecT __attribute__((ext_vector_type(VEC)));
    __shared__ float red[4];
    const int r = blockIdx.x;
    clear_words(zero);
    if (rope.table) write_rope_row(rope, r);
    const T *xr = x + map_row(xmap, seq_len, r) * (int64_t)D;
    const int nvec = D / VEC;
    float v[CH][VEC];
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int i = threadIdx.x + 256 * c;
        if (i < nvec) {
            const vecT t = *(const vecT *)(xr + i * VEC);
#pragma unroll
            for (int j = 0; j < VEC; ++j) { v[c][j] = (float)t[j]; s += v[c][j]; }
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) v[c][j] = 0.f;
        }
    }
    float mu = 0.f;
    if (kind == CASCADE_NORM_LAYERNORM) mu = block_sum_256(s, red) / D;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c)
        if (threadIdx.x + 256 * c < nvec)
#pragma unroll
            for (int j = 0; j < VEC; ++j) { const float d0 = v[c][j] - mu; q += d0 * d0; }
    const float rstd = 1.0f / sqrtf(block_sum_256(q, red) / D + eps);
    T *yr = y + map_row(ymap, seq_len, r) * (int64_t)D;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int i = threadIdx.x + 256 * c;
        if (i < nvec) {
            const vecT g = *(const vecT *)(gain + i * VEC);
            vecT o;
            if (bias) {
                const vecT bb = *(const vecT *)(bias + i * VEC);
#pragma unroll
                for (int j = 0; j < VEC; ++j) o[j] = (T)((v[c][j] - mu) * rstd * (float)g[j] + (float)bb[j]);
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) o[j] = (T)((v[c][j] - mu) * rstd * (float)g[j]);
            }
            *(vecT *)(yr + i * VEC) = o;
        }
    }
}

template <typename T>
static int32_t launch_norm_t(const NormArgs &a, hipStream_t s) {
    constexpr int VEC = 16 / sizeof(T);
    const bool aligned = a.D % VEC == 0 && ((uintptr_t)a.x | (uintptr_t)a.y | (uintptr_t)a.gain | (uintptr_t)a.bias) % 16 == 0;
    const int nvec = a.D / VEC;
    const RopeTableOut rope = {a.rope_table, a.rope_pos, a.rope_seq_len, a.rope_head_dim, a.rope_theta};
    const ZeroWords zero = {a.zero_words, a.n_zero_words};
#define NORM_VEC(CH)                                                                                             \
    hipLaunchKernelGGL((norm_vec_kernel<T, CH>), dim3(a.rows), dim3(256), 0, s, (const T *)a.x, (const T *)a.gain, \
                       (const T *)a.bias, (T *)a.y, a.D, a.kind, a.eps, a.xmap.map, a.ymap.map,                 \
                       a.xmap.map ? a.xmap.seq_len : a.ymap.seq_len, rope, zero)
    if (aligned && nvec <= 256) NORM_VEC(1);
    else if (aligned && nvec <= 512) NORM_VEC(2);
    else if (aligned && nvec <= 1024) NORM_VEC(4);
    else {
        size_t lds = (size_t)a.D * sizeof(float);
        if (lds > 64 * 1024) return CASCADE_EUNSUPPORTED;
        hipLaunchKernelGGL(norm_kernel<T>, dim3(a.rows), dim3(256), lds, s, (const T *)a.x, (const T *)a.gain,
                           (const T *)a.bias, (T *)a.y, a.D, a.kind, a.eps, a.xmap.map, a.ymap.map,
                           a.xmap.map ? a.xmap.seq_len : a.ymap.seq_len, rope, zero);
    }
#undef NORM_VEC
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

int32_t launch_norm(const NormArgs &a, hipStream_t s) {
    if (a.rows == 0) return CASCADE_OK;
    return a.dtype == CASCADE_BF16 ? launch_norm_t<bf16_t>(a, s) : launch_norm_t<float>(a, s);
}

// ---------------------------------------------------------------------------- prefill k, v -> cache slabs
// One workgroup per (kv shard, kv head, sequence); 16-byte pieces, a row of d elements per d*sizeof(T)/16 lanes.
template <typename T>
__global__ __launch_bounds__(256) void kv_to_cache_kernel(KvCacheArgs a) {
    constexpr int VEC = 16 / sizeof(T);
    const int k = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int r0 = a.offsets[k], n = a.offsets[k + 1] - r0;
    if (g == 0 && threadIdx.x == 0) a.shard_len[b * a.n_shards + k] = n;
    const int cpr = a.d / VEC;                              // pieces per row
    const T *act = (const T *)a.act + (int64_t)b * a.N * a.ld;
    T *kc = (T *)a.k_cache + (((int64_t)b * a.Hkv + g) * a.n_shards + k) * (int64_t)a.cap * a.d;
    T *vc = (T *)a.v_cache + (((int64_t)b * a.Hkv + g) * a.n_shards + k) * (int64_t)a.cap * a.d;
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    for (int id = threadIdx.x; id < n * cpr; id += 256) {
        const int i = id / cpr, c = id - i * cpr;
        const int row = a.row_of ? a.row_of[r0 + i] : r0 + i;
        const T *src = act + (int64_t)row * a.ld + g * a.d + c * VEC;
        *(vec_t *)(kc + (int64_t)i * a.d + c * VEC) = *(const vec_t *)(src + a.k_col0);
        *(vec_t *)(vc + (int64_t)i * a.d + c * VEC) = *(const vec_t *)(src + a.v_col0);
    }
}

int32_t launch_kv_to_cache(const KvCacheArgs &a, hipStream_t s) {
    const int vec = a.dtype == CASCADE_BF16 ? 8 : 4;
    if (a.d % vec || a.ld % vec || a.k_col0 % vec || a.v_col0 % vec ||
        ((uintptr_t)a.act | (uintptr_t)a.k_cache | (uintptr_t)a.v_cache) % 16)
        return CASCADE_EUNSUPPORTED;
    if (a.n_shards > 65535 * 32 || a.Hkv > 65535 || a.B > 65535) return CASCADE_EUNSUPPORTED;
    dim3 grid(a.n_shards, a.Hkv, a.B);
    if (a.dtype == CASCADE_BF16) hipLaunchKernelGGL(kv_to_cache_kernel<bf16_t>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(kv_to_cache_kernel<float>, grid, dim3(256), 0, s, a);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

// ---------------------------------------------------------------------------- greedy token
// Lowest index of the largest logit of a row (the CompNode holding the last token turns its logits
// into the next token).  One 1024-thread block per row; a thread walks ascending indices and keeps
// the first maximum it meets, the reductions prefer the lower index among equal values.  NaNs never
// win a comparison; a row of NaNs gives 0.
template <typename T>
__global__ __launch_bounds__(1024) void argmax_rows_kernel(const T *__restrict__ x, int64_t ld, int vocab,
                                                           int32_t *__restrict__ out) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const T *row = x + (int64_t)blockIdx.x * ld;
    float best = -INFINITY;
    int idx = INT32_MAX;
    constexpr int VEC = 16 / sizeof(T);
    if (vocab % VEC == 0 && (((uintptr_t)x | (uintptr_t)(ld * sizeof(T))) % 16) == 0) {
        typedef T vec_t __attribute__((ext_vector_type(VEC)));     // 16-byte pieces, several in flight per thread
        const int nvec = vocab / VEC;
#pragma unroll 4
        for (int c = threadIdx.x; c < nvec; c += 1024) {
            const vec_t pv = *(const vec_t *)(row + (int64_t)c * VEC);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const float v = (float)pv[k];
                if (v > best) { best = v; idx = c * VEC + k; }      // ascending indices: the first maximum stays
            }
        }
    } else {
        for (int i = threadIdx.x; i < vocab; i += 1024) {
            const float v = Elem<T>::load(row + i);
            if (v > best) { best = v; idx = i; }
        }
    }
    auto take = [&](float ov, int oi) {
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    };
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) take(__shfl_xor(best, o, WAVE), __shfl_xor(idx, o, WAVE));
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) take(sv[w], si[w]);
        out[blockIdx.x] = idx == INT32_MAX ? 0 : idx;
    }
}

int32_t launch_argmax_rows(int32_t dtype, const void *x, int64_t ld, int32_t rows, int32_t vocab, int32_t *token_out,
                           hipStream_t s) {
    if (rows == 0) return CASCADE_OK;
    if (dtype == CASCADE_BF16)
        hipLaunchKernelGGL(argmax_rows_kernel<bf16_t>, dim3(rows), dim3(1024), 0, s, (const bf16_t *)x, ld, vocab, token_out);
    else
        hipLaunchKernelGGL(argmax_rows_kernel<float>, dim3(rows), dim3(1024), 0, s, (const float *)x, ld, vocab, token_out);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

// ---------------------------------------------------------------------------- rotary embedding
// Half-split pairing (i, i + d/2), angle = position * theta^(-2i/d); position = the token's own
// position (pos_packed[r mod N]), never the shard-local row number.  One thread per pair.
template <typename T, typename ANG>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ x, int64_t total_pairs, int n_rope_heads,
                                                   int head_dim, int64_t ld, float theta,
                                                   const int32_t *__restrict__ pos_packed, int seq_len) {
    const int half = head_dim >> 1;
    const int64_t pairs_per_row = (int64_t)n_rope_heads * half;
    for (int64_t id = blockIdx.x * 256ll + threadIdx.x; id < total_pairs; id += (int64_t)gridDim.x * 256) {
        int64_t r = id / pairs_per_row;
        int rem = (int)(id - r * pairs_per_row);
        int h = rem / half, i = rem - h * half;
        int pos = pos_packed[(int)(r % seq_len)];
        ANG inv_freq = (ANG)exp2((ANG)(-2.0 * i / head_dim) * (ANG)log2((ANG)theta));
        ANG ang = (ANG)pos * inv_freq;
        ANG sn = sin(ang), cs = cos(ang);
        T *p = x + r * ld + (int64_t)h * head_dim + i;
        ANG a = (ANG)Elem<T>::load(p), b = (ANG)Elem<T>::load(p + half);
        Elem<T>::store(p, (float)(a * cs - b * sn));
        Elem<T>::store(p + half, (float)(b * cs + a * sn));
    }
}

// Vector variant for bf16: one thread rotates 8 consecutive pairs (two 16-byte pieces half a head apart).
// rev[i] = theta^(-2i/d) / (2 pi) comes from the host in double precision, split into two floats.
#define ROPE_MAX_HALF 128
struct RopeFreq {
    float hi[ROPE_MAX_HALF], lo[ROPE_MAX_HALF];
};

__global__ __launch_bounds__(256) void rope_vec_kernel(bf16_t *__restrict__ x, int64_t total_units, int n_rope_heads,
                                                       int head_dim, int64_t ld, RopeFreq freq,
                                                       const int32_t *__restrict__ pos_packed, int seq_len) {
    const int half = head_dim >> 1;
    const int upr = n_rope_heads * (half / 8);                    // units per row
    for (int64_t id = blockIdx.x * 256ll + threadIdx.x; id < total_units; id += (int64_t)gridDim.x * 256) {
        const int64_t r = id / upr;
        const int rem = (int)(id - r * upr);
        const int h = rem / (half / 8), i0 = (rem % (half / 8)) * 8;
        const float pos = (float)pos_packed[(int)(r % seq_len)];  // exact: positions are below 2^24
        bf16_t *p = x + r * ld + (int64_t)h * head_dim + i0;
        const bf16x8 a = *(const bf16x8 *)p, b = *(const bf16x8 *)(p + half);
        bf16x8 oa, ob;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float cs, sn;
            rope_cos_sin(pos, freq.hi[i0 + j], freq.lo[i0 + j], cs, sn);
            const float fa = (float)a[j], fb = (float)b[j];
            oa[j] = (bf16_t)(fa * cs - fb * sn);
            ob[j] = (bf16_t)(fb * cs + fa * sn);
        }
        *(bf16x8 *)p = oa;
        *(bf16x8 *)(p + half) = ob;
    }
}

int32_t launch_rope(const RopeArgs &a, hipStream_t s) {
    int64_t total = (int64_t)a.rows * a.n_rope_heads * (a.head_dim / 2);
    if (total == 0) return CASCADE_OK;
    if (a.dtype == CASCADE_BF16 && (a.head_dim / 2) % 8 == 0 && a.head_dim / 2 <= ROPE_MAX_HALF && a.ld % 8 == 0 &&
        (uintptr_t)a.x % 16 == 0 && a.max_pos < (1 << 24)) {
        const int64_t units = total / 8;
        const int grid = (int)std::min<int64_t>((units + 255) / 256, 1 << 20);
        RopeFreq freq;
        for (int i = 0; i < a.head_dim / 2; ++i) {
            const double rev = pow((double)a.theta, -2.0 * i / a.head_dim) / 6.283185307179586476925;
            freq.hi[i] = (float)rev;
            freq.lo[i] = (float)(rev - (double)freq.hi[i]);
        }
        hipLaunchKernelGGL(rope_vec_kernel, dim3(grid), dim3(256), 0, s, (bf16_t *)a.x, units, a.n_rope_heads,
                           a.head_dim, a.ld, freq, a.pos_packed, a.seq_len);
        CASCADE_HIP_TRY(hipGetLastError());
        return CASCADE_OK;
    }
    int grid = (int)std::min<int64_t>((total + 255) / 256, 65536);
    if (a.dtype == CASCADE_BF16)
        hipLaunchKernelGGL((rope_kernel<bf16_t, float>), dim3(grid), dim3(256), 0, s, (bf16_t *)a.x, total,
                           a.n_rope_heads, a.head_dim, a.ld, a.theta, a.pos_packed, a.seq_len);
    else
        hipLaunchKernelGGL((rope_kernel<float, double>), dim3(grid), dim3(256), 0, s, (float *)a.x, total,
                           a.n_rope_heads, a.head_dim, a.ld, a.theta, a.pos_packed, a.seq_len);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}
