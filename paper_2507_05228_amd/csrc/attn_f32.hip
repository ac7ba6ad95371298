// fp32 partial attention (Algorithm 3) and its fused variant (running merge of Algorithm 4).
// One wavefront owns one (batch, head, packed query row[, kv shard]) and walks the key rows in
// chunks of 64: lane c scores key c (a = scale q.k + s), the row maximum and the sum of
// exponentials are 64-lane reductions, and u~ is accumulated with the lanes spread over the
// head dimension.  Plain fp32 FMA + expf: meant for the fp32 configuration (1e-5 tolerance),
// not for speed.
#include "common.h"
#include "device_utils.h"

#define F32_MAX_D 256

template <bool FUSED>
__global__ __launch_bounds__(256) void attn_f32_kernel(
    const float *__restrict__ q, const float *__restrict__ k, const float *__restrict__ v, int B, int H, int Hkv,
    int d, int N, int S, float scale, int causal, int64_t qs_b, int64_t qs_h, int64_t qs_n, int64_t ks_b,
    int64_t ks_h, int64_t ks_n, const int32_t *__restrict__ q_rowmap, const int32_t *__restrict__ kv_rowmap,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ pos_packed,
    const int32_t *__restrict__ pos_kv, float *__restrict__ m_out,
    float *__restrict__ e_out, float *__restrict__ u_out, int u_mode, float *__restrict__ o_out, int64_t o_ld,
    const int32_t *__restrict__ o_rowmap) {
    __shared__ float qs[4][F32_MAX_D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = blockIdx.x * 4 + wave;
    const int h = blockIdx.y;
    const int b = FUSED ? blockIdx.z : blockIdx.z / S;
    const int kk = FUSED ? 0 : blockIdx.z % S;
    const bool live = r < N;                          // wave-uniform
    const int rr = live ? r : N - 1;
    const int g = h / (H / Hkv);
    const float *qrow = q + b * qs_b + h * qs_h + (int64_t)(q_rowmap ? q_rowmap[rr] : rr) * qs_n;
    for (int i = lane; i < d; i += 64) qs[wave][i] = qrow[i];
    __syncthreads();
    if (!live) return;
    const int pos_q = pos_packed[rr];
    const int c_begin = FUSED ? 0 : offsets[kk];
    const int c_end = FUSED ? N : offsets[kk + 1];
    const float *kb = k + b * ks_b + g * ks_h;
    const float *vb = v + b * ks_b + g * ks_h;

    float m = -INFINITY, e = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = c_begin; c0 < c_end; c0 += 64) {
        const int c = c0 + lane;
        const bool valid = c < c_end;
        const int cc = valid ? c : c_end - 1;
        const int64_t krow = kv_rowmap ? kv_rowmap[cc] : cc;
        float s = -INFINITY;
        if (valid && (!causal || pos_kv[cc] <= pos_q)) {
            const float *kr = kb + krow * ks_n;
            float dot = 0.f;
            for (int i = 0; i < d; ++i) dot = fmaf(qs[wave][i], kr[i], dot);
            s = dot * scale;
        }
        const float cm = wave_max(s);
        if (cm == -INFINITY) continue;                // nothing visible in this chunk (wave-uniform)
        const float m_new = fmaxf(m, cm);
        const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
        const float p = (s == -INFINITY) ? 0.f : expf(s - m_new);
        e = e * alpha + wave_sum(p);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] *= alpha;
        const int nc = min(64, c_end - c0);
        for (int t = 0; t < nc; ++t) {
            const float pt = __shfl(p, t, WAVE);
            if (pt == 0.f) continue;                  // wave-uniform
            const int64_t vrow = __shfl((int)krow, t, WAVE);
            const float *vr = vb + vrow * ks_n;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int i = lane + 64 * j;
                if (i < d) acc[j] = fmaf(pt, vr[i], acc[j]);
            }
        }
        m = m_new;
    }
    if (FUSED) {
        const float inv = e > 0.f ? 1.0f / e : 0.f;
        float *op = o_out + ((int64_t)b * N + (o_rowmap ? o_rowmap[r] : r)) * o_ld + (int64_t)h * d;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int i = lane + 64 * j;
            if (i < d) op[i] = acc[j] * inv;
        }
    } else {
        const int64_t me = (((int64_t)b * H + h) * S + kk) * N + r;
        if (lane == 0) { m_out[me] = m; e_out[me] = e; }
        const float f = (u_mode == CASCADE_U_NORMALISED) ? (e > 0.f ? 1.0f / e : 0.f) : 1.0f;
        float *up = u_out + ((((int64_t)b * S + kk) * H + h) * N + r) * d;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int i = lane + 64 * j;
            if (i < d) up[i] = acc[j] * f;
        }
    }
}

int32_t launch_attn_f32(const cascade_plan *p, const AttnArgs &a, hipStream_t s) {
    if (a.d > F32_MAX_D) return CASCADE_EUNSUPPORTED;
    const cascade_plan *kvp = kv_plan(p);             // key rows walk the key/value partition's packed order
    const int N = p->seq_len, S = kvp->n_shards;
    if (a.H > 65535 || (int64_t)a.B * S > 65535) return CASCADE_EUNSUPPORTED;
    dim3 grid((N + 3) / 4, a.H, a.fused ? a.B : a.B * S);
    const int causal = a.mask_kind == CASCADE_MASK_CAUSAL;
    if (a.fused)
        hipLaunchKernelGGL(attn_f32_kernel<true>, grid, dim3(256), 0, s, (const float *)a.q, (const float *)a.k,
                           (const float *)a.v, a.B, a.H, a.Hkv, a.d, N, S, a.scale, causal, a.qs_b, a.qs_h, a.qs_n,
                           a.ks_b, a.ks_h, a.ks_n, a.q_rowmap, a.kv_rowmap, kvp->offsets_d, p->pos_packed_d, kvp->pos_packed_d,
                           a.m, a.e,
                           a.u, a.u_mode, (float *)a.o, a.o_ld, a.o_rowmap);
    else
        hipLaunchKernelGGL(attn_f32_kernel<false>, grid, dim3(256), 0, s, (const float *)a.q, (const float *)a.k,
                           (const float *)a.v, a.B, a.H, a.Hkv, a.d, N, S, a.scale, causal, a.qs_b, a.qs_h, a.qs_n,
                           a.ks_b, a.ks_h, a.ks_n, a.q_rowmap, a.kv_rowmap, kvp->offsets_d, p->pos_packed_d, kvp->pos_packed_d,
                           a.m, a.e,
                           a.u, a.u_mode, (float *)a.o, a.o_ld, a.o_rowmap);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}
