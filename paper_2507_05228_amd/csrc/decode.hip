// Token-sharded KV-cache decode (Cost Optimizations appendix, "Caching"): the newest token's query
// row against the cached keys / values of every kv shard S_k, giving one partial (m, e, u~) per shard,
// which cascade_lse_merge then combines exactly as in the prefill path (the merge of Algorithm 4).
// Every cached key is at or before the new position, so there is no mask; only the shard lengths.
//
// HBM-bound: each cached K and V row is read once.  WPS wavefronts share one (shard, kv head,
// sequence): 1 for small shards (four shards per workgroup, no LDS, no barrier), 4 for large ones
// (more loads in flight per shard; the four running states are merged through LDS).  The REP query
// heads that share the kv head are processed together so the cache is read once for all of them.
// A row is spread over LPR = d / VEC lanes (16 bytes per lane), so one wavefront instruction reads
// 64 / LPR consecutive rows, fully coalesced, and the rows of the next two steps are requested before
// the arithmetic of the current one.  Scores are reduced over the LPR lanes with xor shuffles; each
// lane group keeps a running (m, e, u~) per head (the same online recurrence as the fused prefill
// kernel); the lane groups of a wavefront are merged with shuffles at the end.
#include <cmath>
#include <type_traits>
#include "common.h"
#include "device_utils.h"

#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f

struct DecodeParams {
    const void *q, *kc, *vc;
    const int32_t *shard_len;
    float *m, *e, *u;
    int32_t B, H, Hkv, S, cap, d;
    float scale_log2;
    int32_t u_mode;
    int32_t per_head;        // 1: one query head per workgroup (kv head = head / rep)
    int32_t rep;
};

// Sum over the LPR lanes that hold one row (LPR a power of two, lane groups aligned).  Inside a 16-lane row
// the exchange is a data-parallel-primitive modifier on the add (no LDS traffic): lanes ^1 and ^2 by quad
// permutes, then the two mirrors (a sum does not care that they reverse instead of swapping halves); wider
// groups finish with cross-row shuffles.  Every lane of the group ends with the total.
template <int LPR>
__device__ __forceinline__ float group_sum(float s) {
    auto dpp_add = [](float v, auto ctrl_tag) {
        constexpr int ctrl = decltype(ctrl_tag)::value;
        return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true));
    };
    if (LPR >= 2) s = dpp_add(s, std::integral_constant<int, 0xB1>());     // quad_perm [1,0,3,2]
    if (LPR >= 4) s = dpp_add(s, std::integral_constant<int, 0x4E>());     // quad_perm [2,3,0,1]
    if (LPR >= 8) s = dpp_add(s, std::integral_constant<int, 0x141>());    // row_half_mirror
    if (LPR >= 16) s = dpp_add(s, std::integral_constant<int, 0x140>());   // row_mirror
#pragma unroll
    for (int o = 16; o < LPR; o <<= 1) s += __shfl_xor(s, o, WAVE);
    return s;
}

template <typename T, int REP, int LPR, int WPS>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeParams p) {
    constexpr int VEC = 16 / sizeof(T);
    constexpr int RPW = 64 / LPR;                          // rows per wavefront instruction
    constexpr int AHEAD = WPS == 1 ? 2 : 1;                // row steps requested ahead of their use
    typedef T vecT __attribute__((ext_vector_type(VEC)));
    __shared__ float red_me[WPS == 1 ? 1 : 4][REP][2];
    extern __shared__ float red_u[];                       // [4][REP][d] when WPS == 4

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, rgrp = lane / LPR;
    const int wsub = wave % WPS;                           // this wavefront's share of the shard's rows
    const int k = blockIdx.x * (4 / WPS) + wave / WPS, b = blockIdx.z;
    if (k >= p.S) return;                                  // uniform over the wavefronts that share a shard
    const int head0 = p.per_head ? blockIdx.y : blockIdx.y * REP;      // first query head handled here
    const int g = p.per_head ? blockIdx.y / p.rep : blockIdx.y;        // kv head
    const int d = p.d;
    const int len = min(p.shard_len[b * p.S + k], p.cap);

    float qf[REP][VEC];
#pragma unroll
    for (int h = 0; h < REP; ++h) {
        const vecT t = *(const vecT *)((const T *)p.q + ((int64_t)b * p.H + head0 + h) * d + sub * VEC);
#pragma unroll
        for (int i = 0; i < VEC; ++i) qf[h][i] = (float)t[i] * p.scale_log2;
    }
    float mrun[REP], erun[REP], acc[REP][VEC];
#pragma unroll
    for (int h = 0; h < REP; ++h) {
        mrun[h] = -INFINITY;
        erun[h] = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[h][i] = 0.f;
    }

    const int64_t base = (((int64_t)b * p.Hkv + g) * p.S + k) * p.cap;
    const T *kc = (const T *)p.kc + base * d + sub * VEC;
    const T *vc = (const T *)p.vc + base * d + sub * VEC;
    const int iters = (len + WPS * RPW - 1) / (WPS * RPW);  // uniform trip count: shuffles stay convergent
    vecT kbuf[AHEAD + 1], vbuf[AHEAD + 1];
    auto row_of = [&](int it) { return (it * WPS + wsub) * RPW + rgrp; };
    auto load_row = [&](int it, vecT &kv, vecT &vv) {
        const int r = row_of(it);
        const int rr = r < len ? r : 0;                    // row 0 exists whenever the loop runs
        kv = *(const vecT *)(kc + (int64_t)rr * d);
        vv = *(const vecT *)(vc + (int64_t)rr * d);
    };
#pragma unroll
    for (int a = 0; a < AHEAD; ++a)
        if (a < iters) load_row(a, kbuf[a], vbuf[a]);
    for (int it0 = 0; it0 < iters; it0 += AHEAD + 1) {
#pragma unroll
        for (int a = 0; a <= AHEAD; ++a) {                 // unrolled so the row buffers stay in registers
            const int it = it0 + a;
            if (it >= iters) break;
            if (it + AHEAD < iters) load_row(it + AHEAD, kbuf[(a + AHEAD) % (AHEAD + 1)], vbuf[(a + AHEAD) % (AHEAD + 1)]);
            const vecT kv = kbuf[a], vv = vbuf[a];
            const bool valid = row_of(it) < len;
#pragma unroll
            for (int h = 0; h < REP; ++h) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < VEC; ++i) s = fmaf(qf[h][i], (float)kv[i], s);
                s = group_sum<LPR>(s);
                if (!valid) s = -INFINITY;
                const float m_new = fmaxf(mrun[h], s);
                const float m_sub = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(mrun[h] - m_sub);
                const float pr = __builtin_amdgcn_exp2f(s - m_sub);
                mrun[h] = m_new;
                erun[h] = erun[h] * alpha + pr;
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[h][i] = acc[h][i] * alpha + pr * (float)vv[i];
            }
        }
    }
    // merge the RPW lane groups of the wavefront (lanes with equal `sub`)
#pragma unroll
    for (int h = 0; h < REP; ++h) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            const float m_o = __shfl_xor(mrun[h], o, WAVE), e_o = __shfl_xor(erun[h], o, WAVE);
            const float m_new = fmaxf(mrun[h], m_o);
            const float m_sub = m_new == -INFINITY ? 0.f : m_new;
            const float a0 = __builtin_amdgcn_exp2f(mrun[h] - m_sub), a1 = __builtin_amdgcn_exp2f(m_o - m_sub);
            erun[h] = erun[h] * a0 + e_o * a1;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[h][i] = acc[h][i] * a0 + __shfl_xor(acc[h][i], o, WAVE) * a1;
            mrun[h] = m_new;
        }
    }
    if (WPS == 1) {                                        // the wavefront owns the shard: write the partial
        if (lane < LPR) {
#pragma unroll
            for (int h = 0; h < REP; ++h) {
                const int head = head0 + h;
                if (lane == 0) {
                    p.m[((int64_t)b * p.H + head) * p.S + k] = mrun[h] * LN2;     // back to the units of a
                    p.e[((int64_t)b * p.H + head) * p.S + k] = erun[h];
                }
                const float f = p.u_mode == CASCADE_U_NORMALISED ? (erun[h] > 0.f ? 1.0f / erun[h] : 0.f) : 1.0f;
                float *up = p.u + (((int64_t)b * p.S + k) * p.H + head) * d + sub * VEC;
#pragma unroll
                for (int i = 0; i < VEC; ++i) up[i] = acc[h][i] * f;
            }
        }
        return;
    }
    // four wavefronts per shard: merge their states through LDS
    if (lane < LPR) {
#pragma unroll
        for (int h = 0; h < REP; ++h) {
            if (lane == 0) { red_me[wave][h][0] = mrun[h]; red_me[wave][h][1] = erun[h]; }
#pragma unroll
            for (int i = 0; i < VEC; ++i) red_u[(wave * REP + h) * d + sub * VEC + i] = acc[h][i];
        }
    }
    __syncthreads();
    for (int id = threadIdx.x; id < REP * d; id += 256) {
        const int h = id / d, i = id - h * d;
        float n = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) n = fmaxf(n, red_me[w][h][0]);
        const float n_sub = n == -INFINITY ? 0.f : n;
        float wsum = 0.f, uu = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = __builtin_amdgcn_exp2f(red_me[w][h][0] - n_sub);
            wsum += c * red_me[w][h][1];
            uu += c * red_u[(w * REP + h) * d + i];
        }
        const int head = head0 + h;
        if (i == 0) {
            p.m[((int64_t)b * p.H + head) * p.S + k] = n * LN2;
            p.e[((int64_t)b * p.H + head) * p.S + k] = wsum;
        }
        const float f = p.u_mode == CASCADE_U_NORMALISED ? (wsum > 0.f ? 1.0f / wsum : 0.f) : 1.0f;
        p.u[(((int64_t)b * p.S + k) * p.H + head) * d + i] = uu * f;
    }
}

template <typename T, int REP>
static int32_t launch_lpr(const DecodeParams &p, int y_dim, hipStream_t s) {
    constexpr int VEC = 16 / sizeof(T);
    const int lpr = p.d / VEC;
    // shards of at least 256 rows get four wavefronts each (measured on MI355X: 5.1 against 3.8 TB/s at
    // 512 rows; at 64-128 rows one wavefront per shard wins, 4.4 against 3.6-4.2 TB/s)
    const bool wide = p.cap >= 256;
    const dim3 grid(wide ? p.S : (p.S + 3) / 4, y_dim, p.B);
    const size_t lds = wide ? (size_t)4 * REP * p.d * sizeof(float) : 0;
    // the merge of the four wavefront states needs 4 * REP * d floats: up to 64 KiB at 8 query heads of 512,
    // above the default dynamic limit, so the limit is raised per kernel instance (once per device)
#define DECODE_LAUNCH(L)                                                                              \
    do {                                                                                              \
        if (wide) {                                                                                   \
            static std::atomic<uint64_t> lds_ready{0};                                                \
            CASCADE_HIP_TRY(ensure_dynamic_lds((const void *)decode_attn_kernel<T, REP, L, 4>, (int)lds, lds_ready)); \
            hipLaunchKernelGGL((decode_attn_kernel<T, REP, L, 4>), grid, dim3(256), lds, s, p);       \
        } else hipLaunchKernelGGL((decode_attn_kernel<T, REP, L, 1>), grid, dim3(256), 0, s, p);      \
    } while (0)
    switch (lpr) {
        case 1: DECODE_LAUNCH(1); break;
        case 2: DECODE_LAUNCH(2); break;
        case 4: DECODE_LAUNCH(4); break;
        case 8: DECODE_LAUNCH(8); break;
        case 16: DECODE_LAUNCH(16); break;
        case 32: DECODE_LAUNCH(32); break;
        case 64: DECODE_LAUNCH(64); break;
        default: return CASCADE_EUNSUPPORTED;
    }
#undef DECODE_LAUNCH
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

template <typename T>
static int32_t launch_rep(DecodeParams p, hipStream_t s) {
    const int rep = p.H / p.Hkv;
    p.rep = rep;
    if (p.H > 65535 || p.B > 65535) return CASCADE_EUNSUPPORTED;
    if (rep == 1 || rep == 2 || rep == 4 || rep == 8) {
        p.per_head = 0;
        switch (rep) {
            case 1: return launch_lpr<T, 1>(p, p.Hkv, s);
            case 2: return launch_lpr<T, 2>(p, p.Hkv, s);
            case 4: return launch_lpr<T, 4>(p, p.Hkv, s);
            default: return launch_lpr<T, 8>(p, p.Hkv, s);
        }
    }
    p.per_head = 1;                                        // other group sizes: one query head per wavefront group
    return launch_lpr<T, 1>(p, p.H, s);
}

extern "C" int32_t cascade_decode_partial_attn(const cascade_attn_desc *d, int32_t batch, int32_t n_shards,
                                               int32_t shard_capacity, const int32_t *shard_len_dev, const void *q,
                                               const void *k_cache, const void *v_cache, float *m, float *e, float *u,
                                               void *stream) {
    if (!d || !shard_len_dev || !q || !k_cache || !v_cache || !m || !e || !u) return CASCADE_EINVAL;
    if (batch <= 0 || n_shards <= 0 || shard_capacity <= 0) return CASCADE_EINVAL;
    if (d->dtype != CASCADE_F32 && d->dtype != CASCADE_BF16) return CASCADE_EUNSUPPORTED;
    if (d->n_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || !(d->scale > 0.f)) return CASCADE_EINVAL;
    if (d->n_heads % d->n_kv_heads) return CASCADE_ESHAPE;
    if (d->u_mode != CASCADE_U_NORMALISED && d->u_mode != CASCADE_U_UNNORMALISED) return CASCADE_EINVAL;
    const int vec = d->dtype == CASCADE_BF16 ? 8 : 4;
    const int lpr = d->head_dim / vec;
    if (d->head_dim % vec || lpr > 64 || (lpr & (lpr - 1))) return CASCADE_EUNSUPPORTED;   // d = vec * 2^j, at most 64 lanes per row
    if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache) % 16) return CASCADE_EUNSUPPORTED;
    DecodeParams p = {};
    p.q = q; p.kc = k_cache; p.vc = v_cache; p.shard_len = shard_len_dev; p.m = m; p.e = e; p.u = u;
    p.B = batch; p.H = d->n_heads; p.Hkv = d->n_kv_heads; p.S = n_shards; p.cap = shard_capacity; p.d = d->head_dim;
    p.scale_log2 = d->scale * LOG2E; p.u_mode = d->u_mode;
    hipStream_t s = (hipStream_t)stream;
    return d->dtype == CASCADE_BF16 ? launch_rep<bf16_t>(p, s) : launch_rep<float>(p, s);
}
