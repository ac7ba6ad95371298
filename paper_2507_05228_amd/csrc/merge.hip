// Log-sum-exp merge of the per-shard partials (the merge steps of Algorithm 4; derivation in the
// Post-Pass subsection):  n = max_k m_k,  w = sum_k exp(m_k - n) e_k,
// o = sum_k exp(m_k - n) e_k u_k / w   (with u~ = e u stored: o = sum_k exp(m_k - n) u~_k / w).
// HBM-bound: one pass over n_shards rows of d floats per (batch, head, query row).
//
// Layout: m, e [B, H, S, N]; u [B, S, H, N, d]; o [B, N, H*d].
// A group of G = d/4 lanes owns one (b, h, r): lane s of the group holds columns 4s..4s+3.
// A wavefront therefore covers 64/G consecutive rows r of the same (b, h); the statistics of a
// row are split over the group's lanes (lane s reads shards s, s+G, ...) and combined with
// xor-shuffles inside the group.
#include "common.h"
#include "device_utils.h"

// The partials are read exactly once: non-temporal loads keep them from displacing other data in the caches
// (measured 101 against 105 us on 562 MB, 8 loads in flight per lane; 4 or 16 are no better).
#define MERGE_UNR 8
#define MERGE_LOAD(p) __builtin_nontemporal_load(p)

template <typename T, int G>
__global__ __launch_bounds__(256) void merge_vec_kernel(const float *__restrict__ m, const float *__restrict__ e,
                                                        const float *__restrict__ u, T *__restrict__ o,
                                                        float *__restrict__ lse, int B, int H, int S, int N,
                                                        int64_t o_ld, const int32_t *__restrict__ omap, int u_mode) {
    constexpr int d = G * 4;
    constexpr int RW = 64 / G;                  // rows per wavefront
    constexpr int RB = RW * 4;                  // rows per block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = lane % G;
    const int r = blockIdx.x * RB + wave * RW + lane / G;
    const int h = blockIdx.y, b = blockIdx.z;
    const bool live = r < N;
    const int rr = live ? r : N - 1;            // clamp: dead lanes repeat the last row and do not store
    const float *mrow = m + ((int64_t)(b * H + h) * S) * N + rr;
    const float *erow = e + ((int64_t)(b * H + h) * S) * N + rr;

    float n = -INFINITY;
    for (int k = s; k < S; k += G) n = fmaxf(n, mrow[(int64_t)k * N]);
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) n = fmaxf(n, __shfl_xor(n, off, WAVE));
    const float n_sub = (n == -INFINITY) ? 0.f : n;

    // Coefficients exp(m_k - n) (times e_k for normalised partials): lane s of the group computes those of shards
    // s, s + G, ... once; the streaming loop below fetches them from that lane, so that it holds nothing but
    // independent 16-byte loads of u (UNR of them in flight per lane) and multiply-adds.
    constexpr int KPL = 4;                      // shards per lane kept in registers: S <= KPL * G on this path
    float w = 0.f;
    float coef[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int k = s + i * G;
        coef[i] = 0.f;
        if (k < S) {
            const float mk = mrow[(int64_t)k * N], ek = erow[(int64_t)k * N];
            const float c = (mk == -INFINITY) ? 0.f : expf(mk - n_sub);
            w += c * ek;
            coef[i] = u_mode == CASCADE_U_NORMALISED ? c * ek : c;
        }
    }
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) w += __shfl_xor(w, off, WAVE);

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const float *ub = u + (((int64_t)b * S * H + h) * N + rr) * d + 4 * s;
    const int64_t ustep = (int64_t)H * N * d;
    const int group0 = lane - s;                // first lane of this row's group
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int kbase = i * G;
        if (kbase >= S) break;
        const int kend = min(G, S - kbase);
        int kk = 0;
        for (; kk + MERGE_UNR <= kend; kk += MERGE_UNR) {
            f32x4 uv[MERGE_UNR];
#pragma unroll
            for (int x = 0; x < MERGE_UNR; ++x) uv[x] = MERGE_LOAD((const f32x4 *)(ub + (int64_t)(kbase + kk + x) * ustep));
#pragma unroll
            for (int x = 0; x < MERGE_UNR; ++x) acc += __shfl(coef[i], group0 + kk + x, WAVE) * uv[x];
        }
        for (; kk < kend; ++kk)
            acc += __shfl(coef[i], group0 + kk, WAVE) * MERGE_LOAD((const f32x4 *)(ub + (int64_t)(kbase + kk) * ustep));
    }
    const float inv = w > 0.f ? 1.0f / w : 0.f;
    acc *= inv;
    if (live) {
        int64_t orow = (int64_t)b * N + (omap ? omap[r] : r);
        T *op = o + orow * o_ld + (int64_t)h * d + 4 * s;
        if constexpr (sizeof(T) == 2) {
            bf16x4 v = {(bf16_t)acc[0], (bf16_t)acc[1], (bf16_t)acc[2], (bf16_t)acc[3]};
            *(bf16x4 *)op = v;
        } else {
            *(f32x4 *)op = acc;
        }
        if (lse && s == 0) lse[((int64_t)b * H + h) * N + r] = w > 0.f ? n + logf(w) : -INFINITY;
    }
}

// Few rows (single-token decode: N = 1): one workgroup per (b, h, r); its 256 / G lane groups take the
// shards round-robin (so many loads are in flight per row) and their partial sums meet in LDS.
template <typename T, int G>
__global__ __launch_bounds__(256) void merge_fewrows_kernel(const float *__restrict__ m, const float *__restrict__ e,
                                                            const float *__restrict__ u, T *__restrict__ o,
                                                            float *__restrict__ lse, int B, int H, int S, int N,
                                                            int64_t o_ld, const int32_t *__restrict__ omap, int u_mode) {
    constexpr int d = G * 4;
    constexpr int NG = 256 / G;                 // lane groups in the workgroup
    __shared__ float red[NG][d + 1];
    const int s = threadIdx.x % G, grp = threadIdx.x / G;
    const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const float *mrow = m + ((int64_t)(b * H + h) * S) * N + r;
    const float *erow = e + ((int64_t)(b * H + h) * S) * N + r;
    float n = -INFINITY;
    for (int k = 0; k < S; ++k) n = fmaxf(n, mrow[(int64_t)k * N]);        // S small values, cached: every lane reads all
    const float n_sub = (n == -INFINITY) ? 0.f : n;
    float w = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const float *ub = u + (((int64_t)b * S * H + h) * N + r) * d + 4 * s;
    const int64_t ustep = (int64_t)H * N * d;
    for (int k = grp; k < S; k += NG) {
        const float mk = mrow[(int64_t)k * N], ek = erow[(int64_t)k * N];
        float c = (mk == -INFINITY) ? 0.f : expf(mk - n_sub);
        w += c * ek;
        if (u_mode == CASCADE_U_NORMALISED) c *= ek;
        acc += c * *(const f32x4 *)(ub + k * ustep);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) red[grp][4 * s + j] = acc[j];
    if (s == 0) red[grp][d] = w;
    __syncthreads();
    if (grp == 0) {
        f32x4 tot = {0.f, 0.f, 0.f, 0.f};
        float wt = 0.f;
#pragma unroll
        for (int gq = 0; gq < NG; ++gq) {
#pragma unroll
            for (int j = 0; j < 4; ++j) tot[j] += red[gq][4 * s + j];
            wt += red[gq][d];
        }
        const float inv = wt > 0.f ? 1.0f / wt : 0.f;
        tot *= inv;
        const int64_t orow = (int64_t)b * N + (omap ? omap[r] : r);
        T *op = o + orow * o_ld + (int64_t)h * d + 4 * s;
        if constexpr (sizeof(T) == 2) {
            bf16x4 v = {(bf16_t)tot[0], (bf16_t)tot[1], (bf16_t)tot[2], (bf16_t)tot[3]};
            *(bf16x4 *)op = v;
        } else {
            *(f32x4 *)op = tot;
        }
        if (lse && s == 0) lse[((int64_t)b * H + h) * N + r] = wt > 0.f ? n + logf(wt) : -INFINITY;
    }
}

// Any d: one wavefront per (b, h, r), lanes stride over the columns.
template <typename T>
__global__ __launch_bounds__(256) void merge_scalar_kernel(const float *__restrict__ m, const float *__restrict__ e,
                                                           const float *__restrict__ u, T *__restrict__ o,
                                                           float *__restrict__ lse, int B, int H, int S, int N, int d,
                                                           int64_t o_ld, const int32_t *__restrict__ omap, int u_mode) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = blockIdx.x * 4 + wave;
    const int h = blockIdx.y, b = blockIdx.z;
    if (r >= N) return;
    const float *mrow = m + ((int64_t)(b * H + h) * S) * N + r;
    const float *erow = e + ((int64_t)(b * H + h) * S) * N + r;
    float n = -INFINITY;
    for (int k = lane; k < S; k += 64) n = fmaxf(n, mrow[(int64_t)k * N]);
    n = wave_max(n);
    const float n_sub = (n == -INFINITY) ? 0.f : n;
    float w = 0.f;
    for (int k = lane; k < S; k += 64) {
        float mk = mrow[(int64_t)k * N];
        w += ((mk == -INFINITY) ? 0.f : expf(mk - n_sub)) * erow[(int64_t)k * N];
    }
    w = wave_sum(w);
    const float inv = w > 0.f ? 1.0f / w : 0.f;
    int64_t orow = (int64_t)b * N + (omap ? omap[r] : r);
    for (int c = lane; c < d; c += 64) {
        float acc = 0.f;
        for (int k = 0; k < S; ++k) {
            float mk = mrow[(int64_t)k * N];
            float cf = (mk == -INFINITY) ? 0.f : expf(mk - n_sub);
            if (u_mode == CASCADE_U_NORMALISED) cf *= erow[(int64_t)k * N];
            acc += cf * u[((((int64_t)b * S + k) * H + h) * N + r) * d + c];
        }
        Elem<T>::store(o + orow * o_ld + (int64_t)h * d + c, acc * inv);
    }
    if (lse && lane == 0) lse[((int64_t)b * H + h) * N + r] = w > 0.f ? n + logf(w) : -INFINITY;
}

template <typename T>
static int32_t launch_merge_t(const MergeArgs &a, hipStream_t s) {
    const int G = a.d / 4;
    const bool vec = a.d % 4 == 0 && (G == 4 || G == 8 || G == 16 || G == 32 || G == 64) &&
                     ((uintptr_t)a.u % 16 == 0) && ((uintptr_t)a.o % (4 * sizeof(T)) == 0) &&
                     (a.o_ld * sizeof(T)) % (4 * sizeof(T)) == 0;
#define MERGE_CASE(GG)                                                                                          \
    case GG: {                                                                                                  \
        constexpr int RB = (64 / GG) * 4;                                                                       \
        if (a.N * 2 <= RB && a.N <= 65535) {           /* mostly idle row slots: one workgroup per row */        \
            hipLaunchKernelGGL((merge_fewrows_kernel<T, GG>), dim3(a.N, a.H, a.B), dim3(256), 0, s, a.m, a.e, a.u, \
                               (T *)a.o, a.lse, a.B, a.H, a.n_shards, a.N, a.o_ld, a.o_rowmap, a.u_mode);       \
            break;                                                                                              \
        }                                                                                                       \
        if (a.n_shards > 4 * GG) { fallback = true; break; }   /* more shards than a lane group keeps coefficients for */ \
        dim3 grid((a.N + RB - 1) / RB, a.H, a.B);                                                               \
        hipLaunchKernelGGL((merge_vec_kernel<T, GG>), grid, dim3(256), 0, s, a.m, a.e, a.u, (T *)a.o, a.lse,    \
                           a.B, a.H, a.n_shards, a.N, a.o_ld, a.o_rowmap, a.u_mode);                            \
        break;                                                                                                  \
    }
    bool fallback = !vec;
    if (vec) {
        switch (G) {
            MERGE_CASE(4) MERGE_CASE(8) MERGE_CASE(16) MERGE_CASE(32) MERGE_CASE(64)
        }
    }
    if (fallback) {
        dim3 grid((a.N + 3) / 4, a.H, a.B);
        hipLaunchKernelGGL(merge_scalar_kernel<T>, grid, dim3(256), 0, s, a.m, a.e, a.u, (T *)a.o, a.lse, a.B, a.H,
                           a.n_shards, a.N, a.d, a.o_ld, a.o_rowmap, a.u_mode);
    }
#undef MERGE_CASE
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

int32_t launch_merge(const MergeArgs &a, hipStream_t s) {
    if (a.B == 0 || a.N == 0 || a.H == 0) return CASCADE_OK;
    if (a.H > 65535 || a.B > 65535) return CASCADE_EUNSUPPORTED;
    return a.dtype == CASCADE_BF16 ? launch_merge_t<bf16_t>(a, s) : launch_merge_t<float>(a, s);
}
