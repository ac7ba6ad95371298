// bf16 partial attention on the gfx950 matrix cores (Algorithm 3) and its fused variant, which
// keeps Algorithm 4's running maximum n, weight sum w and output o in registers while it walks the
// key/value shards (same arithmetic as the post-pass, with the maximum updated online).
//
// Work split: a workgroup of 4 wavefronts owns one tile of packed query rows (never straddling a
// shard) for up to 4 query heads that share one key/value head (GQA: the K/V tile in LDS is reused
// by all of them).  A wavefront owns 32*TQ query rows of one head.
//
// MFMA arrangement (32x32x16 bf16): the score block is computed TRANSPOSED, S^T = K Q^T, so that a
// lane holds ONE query row (column lane%32) and 16 keys of it in its accumulator registers.  Row
// maximum and sum of exponentials are then register-local plus one exchange with lane^32; the
// rescale of the output accumulator is a per-lane multiply.  The second product is
// O^T = V^T P^T: the exponentials go from the accumulator layout straight into the B operand (the
// contraction index is permuted consistently on both operands), and V^T is read from a
// transposed copy of V (built once per call by vtranspose_kernel), so both LDS tiles are read with
// vector loads.
//
// Masking: key visible iff position[key] <= position[query] (original token positions).  Tiles and
// 32x32 sub-blocks whose smallest key position exceeds the largest query position are skipped;
// sub-blocks that are fully visible skip the compare.
#include <climits>
#include <cstdlib>
#include "common.h"
#include "device_utils.h"

#define KV_TILE 64
#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f

struct AttnBf16Params {
    const bf16_t *q, *k, *vt;
    int64_t qs_b, qs_h, qs_n, ks_b, ks_h, ks_n, vts_b, vts_h;
    int32_t npad;
    const int32_t *q_rowmap, *kv_rowmap;
    const CascadeTile *qtiles;
    const CascadeTile *kvtiles;
    const int32_t *kv_shard_first;
    int32_t n_kvtiles;
    const int32_t *pos_packed;
    int32_t B, H, Hkv, N, S;
    float scale_log2;
    int32_t causal, fused, u_mode;
    float *m, *e, *u;
    bf16_t *o;
    int64_t o_ld;
    const int32_t *o_rowmap;
    int32_t hpb;          // heads per workgroup (1, 2 or 4)
};

// ---------------------------------------------------------------------------- V -> V^T (tile order)
// vt[b][g][c][64 t + i] = v[b][g][row(tile t, i)][c] for i < n_rows(t), zero for the padding of a
// ragged tile.  Column 64 t of V^T is therefore 16-byte aligned for every key/value tile t.
template <int D>
__global__ __launch_bounds__(256) void vtranspose_kernel(const bf16_t *__restrict__ v, bf16_t *__restrict__ vt,
                                                         int64_t vs_b, int64_t vs_h, int64_t vs_n, int npad,
                                                         int Hkv, const CascadeTile *__restrict__ kvtiles,
                                                         const int32_t *__restrict__ rowmap) {
    __shared__ bf16_t tile[64][D + 2];
    const int t = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int r0 = kvtiles[t].row_start, nr = kvtiles[t].n_rows;
    const bf16_t *vb = v + b * vs_b + g * vs_h;
    constexpr int CPR = D / 8;
    for (int id = threadIdx.x; id < 64 * CPR; id += 256) {
        int rr = id / CPR, ch = id % CPR;
        bf16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
        if (rr < nr) {
            int r = r0 + rr;
            val = *(const bf16x8 *)(vb + (int64_t)(rowmap ? rowmap[r] : r) * vs_n + ch * 8);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) tile[rr][ch * 8 + i] = val[i];
    }
    __syncthreads();
    bf16_t *ob = vt + ((int64_t)b * Hkv + g) * D * npad + (int64_t)t * 64;
    for (int id = threadIdx.x; id < D * 8; id += 256) {
        int c = id / 8, ch = id % 8;
        bf16x8 val;
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] = tile[ch * 8 + i][c];
        *(bf16x8 *)(ob + (int64_t)c * npad + ch * 8) = val;
    }
}

// ---------------------------------------------------------------------------- attention
template <int D, int TQ>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnBf16Params p) {
    constexpr int K_LD = D + 8;                  // padded K row (elements)
    constexpr int V_LD = KV_TILE + 8;            // padded V^T row
    constexpr int K_ELEMS = KV_TILE * K_LD, V_ELEMS = D * V_LD;
    constexpr int BUF_BYTES = (K_ELEMS + V_ELEMS) * 2 + KV_TILE * 4;
    constexpr int KS = D / 16;                   // k-steps of the score product
    constexpr int DB = D / 32;                   // 32-row blocks of O^T
    constexpr int K_CPR = D / 8;                 // 16-byte chunks per K row
    constexpr int K_PER = KV_TILE * K_CPR / 256;
    constexpr int V_PER = D * 8 / 256;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g2 = lane >> 5;
    const int hpb = p.hpb;
    const int hsel = wave % hpb, rg = wave / hpb;
    const int rep = p.H / p.Hkv;
    const int hblocks = rep / hpb;
    const int b = blockIdx.y / (p.Hkv * hblocks);
    const int gh = blockIdx.y % (p.Hkv * hblocks);
    const int g = gh / hblocks;
    const int h = g * rep + (gh % hblocks) * hpb + hsel;
    const int kk = p.fused ? 0 : blockIdx.z;

    const CascadeTile *qtp = p.qtiles + blockIdx.x;
    struct { int row_start, n_rows, pmax; } qt = {qtp->row_start, qtp->n_rows, qtp->pmax};
    const int wrow0 = rg * 32 * TQ;              // first row of this wavefront inside the q tile

    // ---- query fragments (B operand of S^T = K Q^T): lane holds row l32 of each 32-row block
    bf16x8 qf[TQ][KS];
    int posq[TQ];
    int wq_max[TQ], wq_min[TQ];
    bool row_ok[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        int rloc = wrow0 + 32 * qb + l32;
        row_ok[qb] = rloc < qt.n_rows;
        int r = qt.row_start + (row_ok[qb] ? rloc : qt.n_rows - 1);
        const bf16_t *qp = p.q + b * p.qs_b + h * p.qs_h + (int64_t)(p.q_rowmap ? p.q_rowmap[r] : r) * p.qs_n + g2 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *(const bf16x8 *)(qp + ks * 16);
        posq[qb] = p.pos_packed[r];
        int sub = __builtin_amdgcn_readfirstlane(rg * TQ + qb);          // 32-row granule of the q tile
        wq_max[qb] = sub < 8 ? qtp->sub_max[sub] : INT_MIN;
        wq_min[qb] = sub < 8 ? qtp->sub_min[sub] : INT_MAX;
        wq_max[qb] = __builtin_amdgcn_readfirstlane(wq_max[qb]);
        wq_min[qb] = __builtin_amdgcn_readfirstlane(wq_min[qb]);
    }

    // ---- key/value tile range
    const int t_begin = p.fused ? 0 : p.kv_shard_first[kk];
    const int t_end = p.fused ? p.n_kvtiles : p.kv_shard_first[kk + 1];
    auto next_tile = [&](int t) {                // first tile >= t that some query row of the workgroup can see
        while (t < t_end && p.causal && p.kvtiles[t].pmin > qt.pmax) ++t;
        return t;
    };

    const bf16_t *kbase = p.k + b * p.ks_b + g * p.ks_h;
    const bf16_t *vtbase = p.vt + b * p.vts_b + g * p.vts_h;

    u32x4 rk[K_PER], rv[V_PER];
    int rpos = 0;
    auto issue_loads = [&](const CascadeTile &kt, int tile_col) {
#pragma unroll
        for (int i = 0; i < K_PER; ++i) {
            int id = tid + 256 * i;
            int rr = id / K_CPR, ch = id % K_CPR;
            int r = kt.row_start + min(rr, kt.n_rows - 1);        // rows past the tile repeat the last row; masked later
            rk[i] = *(const u32x4 *)(kbase + (int64_t)(p.kv_rowmap ? p.kv_rowmap[r] : r) * p.ks_n + ch * 8);
        }
#pragma unroll
        for (int i = 0; i < V_PER; ++i) {
            int id = tid + 256 * i;
            int c = id / 8, ch = id % 8;
            rv[i] = *(const u32x4 *)(vtbase + (int64_t)c * p.npad + tile_col + ch * 8);
        }
        if (tid < KV_TILE) rpos = p.pos_packed[kt.row_start + min(tid, kt.n_rows - 1)];
    };
    auto store_lds = [&](int buf) {
        bf16_t *ks = (bf16_t *)(smem + buf * BUF_BYTES);
        bf16_t *vs = ks + K_ELEMS;
        int *ps = (int *)(vs + V_ELEMS);
#pragma unroll
        for (int i = 0; i < K_PER; ++i) {
            int id = tid + 256 * i;
            *(u32x4 *)(ks + (id / K_CPR) * K_LD + (id % K_CPR) * 8) = rk[i];
        }
#pragma unroll
        for (int i = 0; i < V_PER; ++i) {
            int id = tid + 256 * i;
            *(u32x4 *)(vs + (id / 8) * V_LD + (id % 8) * 8) = rv[i];
        }
        if (tid < KV_TILE) ps[tid] = rpos;
    };

    f32x16 oacc[TQ][DB];
    float m_run[TQ], l_run[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
    }

    int t = next_tile(t_begin);
    int buf = 0;
    if (t < t_end) {
        issue_loads(p.kvtiles[t], t * KV_TILE);
        store_lds(0);
    }
    __syncthreads();
    while (t < t_end) {
        const CascadeTile kt = p.kvtiles[t];
        const int tn = next_tile(t + 1);
        if (tn < t_end) issue_loads(p.kvtiles[tn], tn * KV_TILE);

        const bf16_t *ks = (const bf16_t *)(smem + buf * BUF_BYTES);
        const bf16_t *vs = ks + K_ELEMS;
        const int *ps = (const int *)(vs + V_ELEMS);

        // ---- S^T blocks: sacc[qb][kb] = K[kb] Q[qb]^T
        f32x16 sacc[TQ][2];
        bool skip[TQ][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bool any = false;
#pragma unroll
            for (int qb = 0; qb < TQ; ++qb) {
                skip[qb][kb] = (kb * 32 >= kt.n_rows) || (p.causal && kt.sub_min[kb] > wq_max[qb]);
                any |= !skip[qb][kb];
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[qb][kb][r] = 0.f;
            }
            if (!any) continue;
            const bf16_t *kp = ks + (kb * 32 + l32) * K_LD + g2 * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                bf16x8 kf = *(const bf16x8 *)(kp + s * 16);
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    if (!skip[qb][kb])
                        sacc[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][s], sacc[qb][kb], 0, 0, 0);
            }
        }

        // ---- mask, row statistics, exponentials, P^T fragments
#pragma unroll
        for (int qb = 0; qb < TQ; ++qb) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (skip[qb][kb]) continue;
                const bool need_mask = (kb * 32 + 32 > kt.n_rows) || (p.causal && kt.sub_max[kb] > wq_min[qb]);
                if (need_mask) {
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int kv0 = kb * 32 + 8 * r4 + 4 * g2;
                        const int4 pk = *(const int4 *)(ps + kv0);
                        const int pks[4] = {pk.x, pk.y, pk.z, pk.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            bool vis = (kv0 + i < kt.n_rows) && (!p.causal || pks[i] <= posq[qb]);
                            if (!vis) sacc[qb][kb][4 * r4 + i] = -INFINITY;
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[qb][kb][r]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
            const float m_new = fmaxf(m_run[qb], mx * p.scale_log2);
            const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_sub);
            m_run[qb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (skip[qb][kb]) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float pv = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][r], p.scale_log2, -m_sub));
                    sacc[qb][kb][r] = pv;
                    psum += pv;
                }
            }
            l_run[qb] = l_run[qb] * alpha + psum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
        }

        // ---- O^T += V^T P^T.  Step s covers keys 16s..16s+15 of the tile; k-slot (g2, i) of both
        // operands is key 16s + 8(i/4) + 4 g2 + i%4, which is accumulator register 8(s%2)+i of block s/2.
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int kb = s >> 1;
            bool any = false;
            bf16x8 pf[TQ];
#pragma unroll
            for (int qb = 0; qb < TQ; ++qb) {
                any |= !skip[qb][kb];
#pragma unroll
                for (int i = 0; i < 8; ++i) pf[qb][i] = (bf16_t)sacc[qb][kb][8 * (s & 1) + i];
            }
            if (!any) continue;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16_t *vp = vs + (db * 32 + l32) * V_LD + 16 * s + 4 * g2;
                bf16x4 lo = *(const bf16x4 *)vp, hi = *(const bf16x4 *)(vp + 8);
                bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    if (!skip[qb][kb])
                        oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb], oacc[qb][db], 0, 0, 0);
            }
        }

        if (tn < t_end) store_lds(buf ^ 1);
        __syncthreads();
        buf ^= 1;
        t = tn;
    }

    // ---- write-out.  oacc[qb][db][r]: query row 32qb + l32, column 32db + 8(r/4) + 4 g2 + r%4.
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, WAVE);
        if (!row_ok[qb]) continue;
        const int r = qt.row_start + wrow0 + 32 * qb + l32;
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        if (p.fused) {
            bf16_t *op = p.o + ((int64_t)b * p.N + (p.o_rowmap ? p.o_rowmap[r] : r)) * p.o_ld + (int64_t)h * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    bf16x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (bf16_t)(oacc[qb][db][4 * r4 + i] * inv);
                    *(bf16x4 *)(op + 32 * db + 8 * r4 + 4 * g2) = v;
                }
        } else {
            const int64_t me = (((int64_t)b * p.H + h) * p.S + kk) * p.N + r;
            if (g2 == 0) {
                p.m[me] = m_run[qb] * LN2;
                p.e[me] = l_tot;
            }
            const float f = p.u_mode == CASCADE_U_NORMALISED ? inv : 1.0f;
            float *up = p.u + ((((int64_t)b * p.S + kk) * p.H + h) * p.N + r) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = oacc[qb][db][4 * r4 + i] * f;
                    *(f32x4 *)(up + 32 * db + 8 * r4 + 4 * g2) = v;
                }
        }
    }
}

static int32_t npad_of(const cascade_plan *p) { return std::max(1, plan_tiles(p, KV_TILE).count) * KV_TILE; }

size_t attn_bf16_workspace_bytes(const cascade_plan *p, int32_t B, int32_t Hkv, int32_t d) {
    return align_up((size_t)B * Hkv * d * npad_of(p) * 2, 256);
}

template <int D, int TQ>
static int32_t launch_attn_cfg(const cascade_plan *p, const AttnArgs &a, hipStream_t s) {
    const int N = p->seq_len, S = p->n_shards;
    const int rep = a.H / a.Hkv;
    const int hpb = rep % 4 == 0 ? 4 : rep % 2 == 0 ? 2 : 1;
    const int rowgroups = 4 / hpb;
    const int granule = 32 * TQ * rowgroups;                   // 32 .. 256
    const CascadeTileList &ql = plan_tiles(p, granule);
    const CascadeTileList &kl = plan_tiles(p, KV_TILE);
    const int npad = npad_of(p);

    bf16_t *vt = (bf16_t *)a.workspace;
    {
        dim3 grid(kl.count, a.Hkv, a.B);
        hipLaunchKernelGGL(vtranspose_kernel<D>, grid, dim3(256), 0, s, (const bf16_t *)a.v, vt, a.ks_b, a.ks_h,
                           a.ks_n, npad, a.Hkv, kl.dev, a.kv_rowmap);
        CASCADE_HIP_TRY(hipGetLastError());
    }
    AttnBf16Params k;
    k.q = (const bf16_t *)a.q; k.k = (const bf16_t *)a.k; k.vt = vt;
    k.qs_b = a.qs_b; k.qs_h = a.qs_h; k.qs_n = a.qs_n; k.ks_b = a.ks_b; k.ks_h = a.ks_h; k.ks_n = a.ks_n;
    k.vts_b = (int64_t)a.Hkv * D * npad; k.vts_h = (int64_t)D * npad; k.npad = npad;
    k.q_rowmap = a.q_rowmap; k.kv_rowmap = a.kv_rowmap;
    k.qtiles = ql.dev; k.kvtiles = kl.dev; k.kv_shard_first = kl.shard_first; k.n_kvtiles = kl.count;
    k.pos_packed = p->pos_packed_d;
    k.B = a.B; k.H = a.H; k.Hkv = a.Hkv; k.N = N; k.S = S;
    k.scale_log2 = a.scale * LOG2E;
    k.causal = a.mask_kind == CASCADE_MASK_CAUSAL; k.fused = a.fused; k.u_mode = a.u_mode;
    k.m = a.m; k.e = a.e; k.u = a.u; k.o = (bf16_t *)a.o; k.o_ld = a.o_ld; k.o_rowmap = a.o_rowmap;
    k.hpb = hpb;

    constexpr int lds = 2 * ((KV_TILE * (D + 8) + D * (KV_TILE + 8)) * 2 + KV_TILE * 4);
    auto kern = attn_bf16_kernel<D, TQ>;
    static bool attr_set = false;
    if (!attr_set) {
        CASCADE_HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_set = true;
    }
    const int64_t gy = (int64_t)a.B * a.Hkv * (rep / hpb);
    if (gy > 65535 || S > 65535 || ql.count == 0) return ql.count == 0 ? CASCADE_OK : CASCADE_EUNSUPPORTED;
    dim3 grid(ql.count, (unsigned)gy, a.fused ? 1 : S);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, k);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

int32_t launch_attn_bf16(const cascade_plan *p, const AttnArgs &a, hipStream_t s) {
    if (a.d != 64 && a.d != 128) return CASCADE_EUNSUPPORTED;
    if (a.scale <= 0.f) return CASCADE_EUNSUPPORTED;           // the row maximum is taken before scaling
    if (a.workspace_bytes < attn_bf16_workspace_bytes(p, a.B, a.Hkv, a.d) || !a.workspace) return CASCADE_EWORKSPACE;
    if ((a.qs_n | a.qs_h | a.qs_b | a.ks_n | a.ks_h | a.ks_b) % 8 ||
        ((uintptr_t)a.q | (uintptr_t)a.k | (uintptr_t)a.v | (uintptr_t)a.workspace) % 16)
        return CASCADE_EUNSUPPORTED;
    const char *tq = getenv("CASCADE_ATTN_TQ");
    const int TQ = tq ? atoi(tq) : 2;
    if (a.d == 128) return TQ == 1 ? launch_attn_cfg<128, 1>(p, a, s) : launch_attn_cfg<128, 2>(p, a, s);
    return TQ == 1 ? launch_attn_cfg<64, 1>(p, a, s) : launch_attn_cfg<64, 2>(p, a, s);
}
