// C-ABI entry points: argument checks, then the kernels.  No compute happens here.
#include "common.h"

static inline int esize(int dtype) { return dtype == CASCADE_BF16 ? 2 : 4; }
static inline bool dtype_ok(int dtype) { return dtype == CASCADE_BF16 || dtype == CASCADE_F32; }
static inline bool rows_ok(int v) { return v == CASCADE_ROWS_ORIGINAL || v == CASCADE_ROWS_PACKED; }

static RowMap rowmap_for(const cascade_plan *plan, int rows_kind) {
    RowMap m;
    m.map = (rows_kind == CASCADE_ROWS_ORIGINAL && plan) ? plan->perm_d : nullptr;
    m.seq_len = plan ? plan->seq_len : 1;
    return m;
}

static int32_t run_gemm(const GemmArgs &g, hipStream_t s) {
    return g.dtype == CASCADE_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
}

// ---------------------------------------------------------------------------- cascade_shard_gemm
extern "C" int32_t cascade_shard_gemm(const cascade_plan *plan, const cascade_gemm_desc *d, const void *X,
                                      const void *W, const void *W_up, const void *bias, const void *residual,
                                      void *Y, void *stream) {
    if (!d || !X || !W || !Y) return CASCADE_EINVAL;
    if (d->rows < 0 || d->k <= 0 || d->n_out <= 0) return CASCADE_EINVAL;
    if (!dtype_ok(d->dtype)) return CASCADE_EUNSUPPORTED;
    if (!rows_ok(d->x_rows) || !rows_ok(d->y_rows) || !rows_ok(d->res_rows)) return CASCADE_EINVAL;
    const int ep = d->epilogue;
    const bool any_map = d->x_rows == CASCADE_ROWS_ORIGINAL || d->y_rows == CASCADE_ROWS_ORIGINAL ||
                         ((ep & CASCADE_EPI_RESIDUAL) && d->res_rows == CASCADE_ROWS_ORIGINAL);
    if ((any_map || (ep & CASCADE_EPI_ROPE)) && !plan) return CASCADE_EINVAL;
    if ((any_map || (ep & CASCADE_EPI_ROPE)) && (int64_t)plan->batch * plan->seq_len != d->rows) return CASCADE_ESHAPE;
    if ((ep & CASCADE_EPI_SWIGLU) && !W_up) return CASCADE_EINVAL;
    if ((ep & CASCADE_EPI_SWIGLU) && (ep & (CASCADE_EPI_BIAS | CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH)))
        return CASCADE_EUNSUPPORTED;
    if ((ep & CASCADE_EPI_GELU_ERF) && (ep & CASCADE_EPI_GELU_TANH)) return CASCADE_EINVAL;
    if ((ep & CASCADE_EPI_BIAS) && !bias) return CASCADE_EINVAL;
    if ((ep & CASCADE_EPI_RESIDUAL) && !residual) return CASCADE_EINVAL;
    if (ep & CASCADE_EPI_ROPE) {
        if (ep & (CASCADE_EPI_RESIDUAL | CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH | CASCADE_EPI_SWIGLU))
            return CASCADE_EUNSUPPORTED;
        if (d->y_rows != CASCADE_ROWS_PACKED) return CASCADE_EUNSUPPORTED;
        if (d->head_dim <= 0 || d->head_dim % 2 || d->rope_cols < 0 || d->rope_cols % d->head_dim ||
            d->rope_cols > d->n_out || d->rope_theta <= 0.f)
            return CASCADE_EUNSUPPORTED;
    }
    if (X == Y) return CASCADE_EINVAL;
    if (residual == Y && d->y_rows != d->res_rows) return CASCADE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    GemmArgs g = {};
    g.dtype = d->dtype; g.M = d->rows; g.N = d->n_out; g.K = d->k;
    g.X = X; g.W[0] = W; g.W[1] = g.W[2] = nullptr;
    g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = d->n_out;
    g.bias[0] = (ep & CASCADE_EPI_BIAS) ? bias : nullptr;
    g.W_up = W_up; g.residual = residual; g.Y = Y;
    g.ldx = d->k; g.ldy = d->n_out; g.ldres = d->n_out;
    g.xmap = rowmap_for(plan, d->x_rows); g.ymap = rowmap_for(plan, d->y_rows); g.rmap = rowmap_for(plan, d->res_rows);
    g.epilogue = ep & ~CASCADE_EPI_ROPE;
    int32_t st = run_gemm(g, s);
    if (st != CASCADE_OK) return st;
    if ((ep & CASCADE_EPI_ROPE) && d->rope_cols > 0) {
        RopeArgs r = {};
        r.dtype = d->dtype; r.rows = d->rows; r.seq_len = plan->seq_len;
        r.n_rope_heads = d->rope_cols / d->head_dim; r.head_dim = d->head_dim; r.ld = d->n_out;
        r.theta = d->rope_theta; r.pos_packed = plan->pos_packed_d; r.x = Y; r.max_pos = plan->max_abs_pos;
        st = launch_rope(r, s);
    }
    return st;
}

// ---------------------------------------------------------------------------- attention ops
static int32_t check_attn_desc(const cascade_plan *plan, const cascade_attn_desc *d) {
    if (!plan || !d) return CASCADE_EINVAL;
    if (!dtype_ok(d->dtype)) return CASCADE_EUNSUPPORTED;
    if (d->n_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0) return CASCADE_EINVAL;
    if (d->n_heads % d->n_kv_heads) return CASCADE_ESHAPE;
    if (!rows_ok(d->row_layout)) return CASCADE_EINVAL;
    if (d->u_mode != CASCADE_U_NORMALISED && d->u_mode != CASCADE_U_UNNORMALISED) return CASCADE_EINVAL;
    if (d->dtype == CASCADE_BF16 && d->head_dim != 64 && d->head_dim != 128) return CASCADE_EUNSUPPORTED;
    if (d->dtype == CASCADE_F32 && d->head_dim > 256) return CASCADE_EUNSUPPORTED;
    return CASCADE_OK;
}

extern "C" size_t cascade_partial_attn_workspace_bytes(const cascade_plan *plan, const cascade_attn_desc *d) {
    if (check_attn_desc(plan, d) != CASCADE_OK) return 0;
    if (d->dtype != CASCADE_BF16) return 0;
    return attn_bf16_workspace_bytes(plan, plan->batch, d->n_kv_heads, d->head_dim);
}

static void fill_strides(const cascade_plan *plan, const cascade_attn_desc *d, AttnArgs &a) {
    const int64_t N = plan->seq_len, dd = d->head_dim;
    a.qs_n = d->q_stride_n ? d->q_stride_n : dd;
    a.qs_h = d->q_stride_h ? d->q_stride_h : N * dd;
    a.qs_b = d->q_stride_b ? d->q_stride_b : (int64_t)d->n_heads * N * dd;
    a.ks_n = d->kv_stride_n ? d->kv_stride_n : dd;
    a.ks_h = d->kv_stride_h ? d->kv_stride_h : N * dd;
    a.ks_b = d->kv_stride_b ? d->kv_stride_b : (int64_t)d->n_kv_heads * N * dd;
}

extern "C" int32_t cascade_partial_attn(const cascade_plan *plan, const cascade_attn_desc *d, const void *q,
                                        const void *k, const void *v, float *m, float *e, float *u, void *workspace,
                                        size_t workspace_bytes, void *stream) {
    int32_t st = check_attn_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!q || !k || !v || !m || !e || !u) return CASCADE_EINVAL;
    AttnArgs a = {};
    a.dtype = d->dtype; a.B = plan->batch; a.H = d->n_heads; a.Hkv = d->n_kv_heads; a.d = d->head_dim;
    a.scale = d->scale; a.mask_kind = plan->mask_kind;
    a.q = q; a.k = k; a.v = v;
    fill_strides(plan, d, a);
    // q rows follow the row partition, k/v rows the key/value partition (the same unless the plan has both)
    a.q_rowmap = d->row_layout == CASCADE_ROWS_ORIGINAL ? plan->perm_d : nullptr;
    a.kv_rowmap = d->row_layout == CASCADE_ROWS_ORIGINAL ? kv_plan(plan)->perm_d : plan->kv_to_row_d;
    a.fused = 0; a.u_mode = d->u_mode; a.m = m; a.e = e; a.u = u;
    a.workspace = workspace; a.workspace_bytes = workspace_bytes;
    hipStream_t s = (hipStream_t)stream;
    return d->dtype == CASCADE_BF16 ? launch_attn_bf16(plan, a, s) : launch_attn_f32(plan, a, s);
}

// ---------------------------------------------------------------------------- partial attention without a workspace
// For callers that cannot allocate (HIP graph capture, tight serving loops): the scratch memory the bf16
// kernels need (V^T in tile order, K gathered into packed order) lives in a static device array of this
// code object instead of a caller's workspace.  Every GPU the library runs on holds its own copy of the
// array at its own address, looked up once per device.
static __device__ __align__(256) unsigned char scratch[CASCADE_STATIC_SCRATCH_BYTES];

static int32_t static_scratch_for_current_device(void **out) {
    constexpr int MAX_DEV = 64;
    static std::atomic<void *> ptrs[MAX_DEV];
    int dev = 0;
    CASCADE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEV) return CASCADE_EUNSUPPORTED;
    void *p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {                                      // the address is per device and fixed: a racing first call stores the same value
        CASCADE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return CASCADE_EHIP;
        ptrs[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return CASCADE_OK;
}

extern "C" int32_t cascade_partial_attn_static(const cascade_plan *plan, const cascade_attn_desc *d, const void *q,
                                               const void *k, const void *v, float *m, float *e, float *u,
                                               void *stream) {
    int32_t st = check_attn_desc(plan, d);
    if (st != CASCADE_OK) return st;
    const size_t need = cascade_partial_attn_workspace_bytes(plan, d);
    if (need > (size_t)CASCADE_STATIC_SCRATCH_BYTES) return CASCADE_EWORKSPACE;
    void *ws = nullptr;
    if (need) {
        st = static_scratch_for_current_device(&ws);
        if (st != CASCADE_OK) return st;
    }
    return cascade_partial_attn(plan, d, q, k, v, m, e, u, ws, need ? (size_t)CASCADE_STATIC_SCRATCH_BYTES : 0, stream);
}

extern "C" int32_t cascade_lse_merge(const cascade_plan *plan, const cascade_attn_desc *d, const float *m,
                                     const float *e, const float *u, void *o, float *lse_out, void *stream) {
    int32_t st = check_attn_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!m || !e || !u || !o) return CASCADE_EINVAL;
    MergeArgs a = {};
    a.dtype = d->dtype; a.B = plan->batch; a.H = d->n_heads; a.d = d->head_dim; a.n_shards = kv_plan(plan)->n_shards;
    a.N = plan->seq_len; a.u_mode = d->u_mode; a.m = m; a.e = e; a.u = u; a.o = o;
    a.o_ld = (int64_t)d->n_heads * d->head_dim;
    a.o_rowmap = d->row_layout == CASCADE_ROWS_ORIGINAL ? plan->perm_d : nullptr;
    a.lse = lse_out;
    return launch_merge(a, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------- whole layer
struct LayerWs {
    size_t x, qkv, ao, h1, act, attn_ws, m, e, u, rope, sk_partial, sk_sync, total;
    size_t attn_ws_bytes, sk_partial_bytes;
};

static LayerWs layer_ws(const cascade_plan *plan, const cascade_layer_desc *d) {
    LayerWs w = {};
    const size_t es = esize(d->dtype);
    const size_t T = (size_t)plan->batch * plan->seq_len;
    const size_t QW = (size_t)(d->n_heads + 2 * d->n_kv_heads) * d->head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    w.x = take(T * d->d_model * es);
    w.qkv = take(T * QW * es);
    w.ao = take(T * (size_t)d->n_heads * d->head_dim * es);
    w.h1 = take(T * d->d_model * es);
    w.act = take(T * (size_t)d->d_ff * es);
    w.attn_ws_bytes = d->dtype == CASCADE_BF16 ? attn_bf16_workspace_bytes(plan, plan->batch, d->n_kv_heads, d->head_dim) : 0;
    w.attn_ws = take(w.attn_ws_bytes);
    w.rope = take(d->rope && d->dtype == CASCADE_BF16 ? T * (size_t)d->head_dim * 4 : 0);   // cos | sin per row
    // o projection and FFN down as split reductions, where their shape asks for it (same output shape, two K)
    w.sk_partial_bytes = 0;
    if (d->dtype == CASCADE_BF16 && T <= (size_t)INT32_MAX)
        w.sk_partial_bytes = std::max(gemm_bf16_splitk_bytes((int32_t)T, d->d_model, d->n_heads * d->head_dim),
                                      gemm_bf16_splitk_bytes((int32_t)T, d->d_model, d->d_ff));
    w.sk_partial = take(w.sk_partial_bytes);
    w.sk_sync = take(w.sk_partial_bytes ? GEMM_SPLITK_SYNC_WORDS * 4 : 0);
    if (d->attn_mode == CASCADE_ATTN_MATERIALISED) {
        const size_t me = (size_t)plan->batch * d->n_heads * kv_plan(plan)->n_shards * plan->seq_len * 4;
        w.m = take(me);
        w.e = take(me);
        w.u = take(me * d->head_dim);
    }
    w.total = off;
    return w;
}

static int32_t check_layer_desc(const cascade_plan *plan, const cascade_layer_desc *d) {
    if (!plan || !d) return CASCADE_EINVAL;
    if (!dtype_ok(d->dtype)) return CASCADE_EUNSUPPORTED;
    if (d->d_model <= 0 || d->n_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->d_ff <= 0)
        return CASCADE_EINVAL;
    if (d->n_heads % d->n_kv_heads) return CASCADE_ESHAPE;
    if (d->norm_kind != CASCADE_NORM_LAYERNORM && d->norm_kind != CASCADE_NORM_RMSNORM) return CASCADE_EINVAL;
    if (d->act != CASCADE_ACT_GELU_ERF && d->act != CASCADE_ACT_GELU_TANH && d->act != CASCADE_ACT_SWIGLU)
        return CASCADE_EINVAL;
    if (d->attn_mode != CASCADE_ATTN_FUSED && d->attn_mode != CASCADE_ATTN_MATERIALISED) return CASCADE_EINVAL;
    if (!rows_ok(d->io_rows)) return CASCADE_EINVAL;
    if (d->norm_placement != CASCADE_NORM_PRE && d->norm_placement != CASCADE_NORM_POST) return CASCADE_EINVAL;
    if (d->rope != 0 && d->rope != 1) return CASCADE_EUNSUPPORTED;
    if (d->rope && (d->head_dim % 2 || d->rope_theta <= 0.f)) return CASCADE_EUNSUPPORTED;
    if (d->dtype == CASCADE_BF16) {
        if (d->head_dim != 64 && d->head_dim != 128) return CASCADE_EUNSUPPORTED;
        if (d->d_model % 8 || d->d_ff % 8) return CASCADE_EUNSUPPORTED;
    } else if (d->head_dim > 256) return CASCADE_EUNSUPPORTED;
    return CASCADE_OK;
}

extern "C" size_t cascade_layer_workspace_bytes(const cascade_plan *plan, const cascade_layer_desc *d) {
    if (check_layer_desc(plan, d) != CASCADE_OK) return 0;
    return layer_ws(plan, d).total;
}

extern "C" int32_t cascade_layer_partials(const cascade_plan *plan, const cascade_layer_desc *d, void *workspace,
                                          float **m, float **e, float **u) {
    int32_t st = check_layer_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!workspace || d->attn_mode != CASCADE_ATTN_MATERIALISED) return CASCADE_EINVAL;
    LayerWs w = layer_ws(plan, d);
    char *base = (char *)workspace;
    if (m) *m = (float *)(base + w.m);
    if (e) *e = (float *)(base + w.e);
    if (u) *u = (float *)(base + w.u);
    return CASCADE_OK;
}

extern "C" int32_t cascade_layer_attention_output(const cascade_plan *plan, const cascade_layer_desc *d,
                                                  void *workspace, void **o) {
    int32_t st = check_layer_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!workspace || !o) return CASCADE_EINVAL;
    *o = (char *)workspace + layer_ws(plan, d).ao;
    return CASCADE_OK;
}

extern "C" size_t cascade_workspace_bytes(const cascade_plan *plan, const void *desc, int32_t op, int32_t flags) {
    switch (op) {
        case CASCADE_OP_PARTIAL_ATTN: return cascade_partial_attn_workspace_bytes(plan, (const cascade_attn_desc *)desc);
        case CASCADE_OP_LAYER_FORWARD: return cascade_layer_workspace_bytes(plan, (const cascade_layer_desc *)desc);
        case CASCADE_OP_LAYER_STACK:
            return cascade_layer_stack_workspace_bytes(plan, (const cascade_layer_desc *)desc, flags);
        case CASCADE_OP_LM_HEAD: return cascade_lm_head_workspace_bytes(plan, (const cascade_lm_head_desc *)desc);
        default: return 0;                         // shard GEMM, LSE merge, decode, norm: no workspace
    }
}

extern "C" int32_t cascade_norm(int32_t dtype, int32_t rows, int32_t d_model, int32_t norm_kind, float eps,
                                const void *x, const void *gain, const void *bias, void *y, void *stream) {
    if (!x || !gain || !y || rows < 0 || d_model <= 0) return CASCADE_EINVAL;
    if (!dtype_ok(dtype)) return CASCADE_EUNSUPPORTED;
    if (norm_kind != CASCADE_NORM_LAYERNORM && norm_kind != CASCADE_NORM_RMSNORM) return CASCADE_EINVAL;
    NormArgs n = {};
    n.dtype = dtype; n.rows = rows; n.D = d_model; n.kind = norm_kind; n.eps = eps;
    n.x = x; n.gain = gain; n.bias = bias; n.y = y;
    n.xmap.map = n.ymap.map = nullptr; n.xmap.seq_len = n.ymap.seq_len = 1;
    return launch_norm(n, (hipStream_t)stream);
}

extern "C" int32_t cascade_layer_kv_to_cache(const cascade_plan *plan, const cascade_layer_desc *d,
                                             const void *workspace, void *k_cache, void *v_cache,
                                             int32_t shard_capacity, int32_t *shard_len_dev, void *stream) {
    int32_t st = check_layer_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!workspace || !k_cache || !v_cache || !shard_len_dev || shard_capacity <= 0) return CASCADE_EINVAL;
    const cascade_plan *kvp = kv_plan(plan);
    for (int k = 0; k < kvp->n_shards; ++k)
        if (kvp->offsets_h[k + 1] - kvp->offsets_h[k] > shard_capacity) return CASCADE_ESHAPE;
    const LayerWs w = layer_ws(plan, d);
    KvCacheArgs a = {};
    a.dtype = d->dtype; a.B = plan->batch; a.N = plan->seq_len; a.Hkv = d->n_kv_heads; a.d = d->head_dim;
    a.n_shards = kvp->n_shards; a.cap = shard_capacity;
    a.act = (const char *)workspace + w.qkv;
    a.ld = (int64_t)(d->n_heads + 2 * d->n_kv_heads) * d->head_dim;
    a.k_col0 = d->n_heads * d->head_dim;
    a.v_col0 = (d->n_heads + d->n_kv_heads) * d->head_dim;
    a.offsets = kvp->offsets_d;
    a.row_of = plan->kv ? plan->kv_to_row_d : nullptr;
    a.k_cache = k_cache; a.v_cache = v_cache; a.shard_len = shard_len_dev;
    return launch_kv_to_cache(a, (hipStream_t)stream);
}

// in_rows / out_rows: row order of h_in / h_out (a layer stack keeps packed order between layers)
static int32_t layer_forward_impl(const cascade_plan *plan, const cascade_layer_desc *d,
                                  const cascade_layer_weights *w, const void *h_in, void *h_out,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  void *const *events, int32_t n_events, int32_t in_rows, int32_t out_rows) {
    int32_t st = check_layer_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!w || !h_in || !h_out || h_in == h_out) return CASCADE_EINVAL;
    if (!w->wq || !w->wk || !w->wv || !w->wo || !w->w_up || !w->w_down || !w->norm1_g || !w->norm2_g)
        return CASCADE_EINVAL;
    if (d->act == CASCADE_ACT_SWIGLU && !w->w_gate) return CASCADE_EINVAL;
    const LayerWs ws = layer_ws(plan, d);
    if (!workspace || workspace_bytes < ws.total) return CASCADE_EWORKSPACE;
    if ((uintptr_t)workspace % 256) return CASCADE_EWORKSPACE;

    hipStream_t s = (hipStream_t)stream;
    int stage = 0;
    auto mark = [&]() -> int32_t {               // optional stage boundary for measurement
        if (events && stage < n_events && events[stage]) {
            hipError_t e = hipEventRecord((hipEvent_t)events[stage], s);
            if (e != hipSuccess) { cascade_set_hip_error(e); return CASCADE_EHIP; }
        }
        ++stage;
        return CASCADE_OK;
    };
    char *base = (char *)workspace;
    const int T = plan->batch * plan->seq_len, N = plan->seq_len;
    const int D = d->d_model, H = d->n_heads, Hkv = d->n_kv_heads, hd = d->head_dim, f = d->d_ff;
    const int QW = (H + 2 * Hkv) * hd;
    const int es = esize(d->dtype);
    void *x = base + ws.x, *qkv = base + ws.qkv, *ao = base + ws.ao, *h1 = base + ws.h1, *act = base + ws.act;
    const RowMap in_map = rowmap_for(plan, in_rows), out_map = rowmap_for(plan, out_rows);
    const RowMap packed = rowmap_for(plan, CASCADE_ROWS_PACKED);
    const bool post = d->norm_placement == CASCADE_NORM_POST;

    // 1. pre-pass: norm (with the gather into packed order), q/k/v projection, rotary embedding (Algorithm 2).
    //    A post-norm block has no norm here: the projection gathers h_in itself.
    if ((st = mark()) != CASCADE_OK) return st;                                   // event 0: start
    GemmArgs g = {};
    g.dtype = d->dtype; g.M = T; g.N = QW; g.K = D; g.X = post ? h_in : x;
    g.W[0] = w->wq; g.W[1] = w->wk; g.W[2] = w->wv;
    g.seg_end[0] = H * hd; g.seg_end[1] = (H + Hkv) * hd; g.seg_end[2] = QW;
    g.bias[0] = w->bq; g.bias[1] = w->bk; g.bias[2] = w->bv;
    {   // q, k, v weights stored back to back (a fused [QW, D] matrix) are one segment: tiles may then
        // straddle the q | k | v boundaries, which lets the tile width be chosen freely
        const char *q0 = (const char *)w->wq, *k0 = (const char *)w->wk, *v0 = (const char *)w->wv;
        const bool w_contig = k0 == q0 + (size_t)H * hd * D * es && v0 == k0 + (size_t)Hkv * hd * D * es;
        const char *bq = (const char *)w->bq, *bk = (const char *)w->bk, *bv = (const char *)w->bv;
        const bool b_contig = (!bq && !bk && !bv) ||
                              (bq && bk == bq + (size_t)H * hd * es && bv == bk + (size_t)Hkv * hd * es);
        if (w_contig && b_contig) g.seg_end[0] = g.seg_end[1] = QW;
    }
    g.epilogue = (w->bq || w->bk || w->bv) ? CASCADE_EPI_BIAS : 0;
    g.Y = qkv; g.ldx = D; g.ldy = QW; g.xmap = post ? in_map : packed; g.ymap = g.rmap = packed;
    // Rotary embedding: in the projection's epilogue when that kernel can do it (bf16, pre-norm: the norm kernel
    // then writes every row's cos | sin table on the side), else as a pass of its own over q and k.
    g.rope_cols = (H + Hkv) * hd; g.rope_head_dim = hd;
    const bool rope_fused = d->rope && !post && d->dtype == CASCADE_BF16 && plan->max_abs_pos < (1 << 24) &&
                            gemm_bf16_rope_fusable(g);
    // The split-reduction GEMMs count on flag words that a norm launch of this call has cleared before them.
    bool sk_ready = false;
    auto clear_sk_sync = [&](NormArgs &n) {
        if (!ws.sk_partial_bytes) return;
        n.zero_words = (uint32_t *)(base + ws.sk_sync); n.n_zero_words = GEMM_SPLITK_SYNC_WORDS;
        sk_ready = true;
    };
    auto offer_splitk = [&](GemmArgs &ga) {
        if (!sk_ready) return;
        ga.sk_partial = (float *)(base + ws.sk_partial); ga.sk_partial_bytes = ws.sk_partial_bytes;
        ga.sk_sync = (uint32_t *)(base + ws.sk_sync);
    };
    if (!post) {
        NormArgs n1 = {d->dtype, T, D, d->norm_kind, d->norm_eps, h_in, w->norm1_g, w->norm1_b, x, in_map, packed};
        clear_sk_sync(n1);
        if (rope_fused) {
            n1.rope_table = (float *)(base + ws.rope); n1.rope_pos = plan->pos_packed_d; n1.rope_seq_len = N;
            n1.rope_head_dim = hd; n1.rope_theta = d->rope_theta;
        }
        if ((st = launch_norm(n1, s)) != CASCADE_OK) return st;
    }
    if ((st = mark()) != CASCADE_OK) return st;                                   // 1: gather + norm1
    if (rope_fused) g.rope_table = (const float *)(base + ws.rope);
    if ((st = run_gemm(g, s)) != CASCADE_OK) return st;
    if ((st = mark()) != CASCADE_OK) return st;                                   // 2: qkv GEMM
    if (d->rope && !rope_fused) {
        RopeArgs r = {d->dtype, T, N, H + Hkv, hd, QW, d->rope_theta, plan->pos_packed_d, qkv, plan->max_abs_pos};
        if ((st = launch_rope(r, s)) != CASCADE_OK) return st;
    }
    if ((st = mark()) != CASCADE_OK) return st;                                   // 3: rotary embedding

    // 2. attention-pass on every (j, k) pair and post-pass merge (Algorithms 3 and 4)
    AttnArgs a = {};
    a.dtype = d->dtype; a.B = plan->batch; a.H = H; a.Hkv = Hkv; a.d = hd; a.scale = d->scale;
    a.mask_kind = plan->mask_kind;
    a.q = qkv; a.k = (char *)qkv + (size_t)H * hd * es; a.v = (char *)qkv + (size_t)(H + Hkv) * hd * es;
    a.qs_b = a.ks_b = (int64_t)N * QW; a.qs_h = a.ks_h = hd; a.qs_n = a.ks_n = QW;
    a.u_mode = CASCADE_U_UNNORMALISED;
    a.kv_rowmap = plan->kv_to_row_d;                                              // null unless S differs from R
    a.workspace = base + ws.attn_ws; a.workspace_bytes = ws.attn_ws_bytes;
    a.o = ao; a.o_ld = (int64_t)H * hd;
    if (d->attn_mode == CASCADE_ATTN_FUSED) {
        a.fused = 1;
        st = d->dtype == CASCADE_BF16 ? launch_attn_bf16(plan, a, s) : launch_attn_f32(plan, a, s);
        if (st != CASCADE_OK) return st;
        if ((st = mark()) != CASCADE_OK) return st;                               // 4: attention
        if ((st = mark()) != CASCADE_OK) return st;                               // 5: (no separate merge)
    } else {
        a.fused = 0;
        a.m = (float *)(base + ws.m); a.e = (float *)(base + ws.e); a.u = (float *)(base + ws.u);
        st = d->dtype == CASCADE_BF16 ? launch_attn_bf16(plan, a, s) : launch_attn_f32(plan, a, s);
        if (st != CASCADE_OK) return st;
        if ((st = mark()) != CASCADE_OK) return st;                               // 4: partial attention
        MergeArgs mg = {d->dtype, plan->batch, H, hd, kv_plan(plan)->n_shards, N, CASCADE_U_UNNORMALISED,
                        a.m, a.e, a.u, ao, (int64_t)H * hd, nullptr, nullptr};
        if ((st = launch_merge(mg, s)) != CASCADE_OK) return st;
        if ((st = mark()) != CASCADE_OK) return st;                               // 5: LSE merge
    }

    // 3. o projection + residual (the projection that closes Algorithm 4, the residual of Algorithm 1's last step)
    g = {};
    g.dtype = d->dtype; g.M = T; g.N = D; g.K = H * hd; g.X = ao; g.W[0] = w->wo;
    g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = D;
    // pre-norm: h1 = h + o Wo^T, then x = norm2(h1) feeds the MLP.
    // post-norm: x = h + o Wo^T, then h1 = norm1(x) is both the MLP input and its residual.
    g.bias[0] = w->bo; g.residual = h_in; g.Y = post ? x : h1;
    g.ldx = H * hd; g.ldy = D; g.ldres = D;
    g.xmap = g.ymap = packed; g.rmap = in_map;
    g.epilogue = CASCADE_EPI_RESIDUAL | (w->bo ? CASCADE_EPI_BIAS : 0);
    offer_splitk(g);
    if ((st = run_gemm(g, s)) != CASCADE_OK) return st;
    if ((st = mark()) != CASCADE_OK) return st;                                   // 6: o projection + residual

    // 4. MLP: norm, up (+ gate) projection with the activation, down projection + residual,
    //    scattered back to the caller's row order
    NormArgs n2 = {d->dtype, T, D, d->norm_kind, d->norm_eps, post ? x : h1, post ? w->norm1_g : w->norm2_g,
                   post ? w->norm1_b : w->norm2_b, post ? h1 : x, packed, packed};
    clear_sk_sync(n2);
    if ((st = launch_norm(n2, s)) != CASCADE_OK) return st;
    if ((st = mark()) != CASCADE_OK) return st;                                   // 7: norm before the MLP
    g = {};
    g.dtype = d->dtype; g.M = T; g.N = f; g.K = D; g.X = post ? h1 : x;
    g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = f;
    g.Y = act; g.ldx = D; g.ldy = f; g.xmap = g.ymap = g.rmap = packed;
    if (d->act == CASCADE_ACT_SWIGLU) {
        g.W[0] = w->w_gate; g.W_up = w->w_up; g.epilogue = CASCADE_EPI_SWIGLU;
    } else {
        g.W[0] = w->w_up; g.bias[0] = w->b_up;
        g.epilogue = (d->act == CASCADE_ACT_GELU_ERF ? CASCADE_EPI_GELU_ERF : CASCADE_EPI_GELU_TANH) |
                     (w->b_up ? CASCADE_EPI_BIAS : 0);
    }
    if ((st = run_gemm(g, s)) != CASCADE_OK) return st;
    if ((st = mark()) != CASCADE_OK) return st;                                   // 8: FFN up (+ gate) GEMM
    g = {};
    g.dtype = d->dtype; g.M = T; g.N = D; g.K = f; g.X = act; g.W[0] = w->w_down;
    g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = D;
    g.bias[0] = w->b_down; g.residual = h1; g.Y = post ? x : h_out;
    g.ldx = f; g.ldy = D; g.ldres = D;
    g.xmap = g.rmap = packed; g.ymap = post ? packed : out_map;
    g.epilogue = CASCADE_EPI_RESIDUAL | (w->b_down ? CASCADE_EPI_BIAS : 0);
    offer_splitk(g);
    if ((st = run_gemm(g, s)) != CASCADE_OK) return st;
    if (post) {                                                                   // closing norm, with the scatter
        NormArgs n3 = {d->dtype, T, D, d->norm_kind, d->norm_eps, x, w->norm2_g, w->norm2_b, h_out, packed, out_map};
        if ((st = launch_norm(n3, s)) != CASCADE_OK) return st;
    }
    return mark();                                                                // 9: FFN down + residual (+ norm) + scatter
}

// ---------------------------------------------------------------------------- layer stack
// Single Layer Pipeline subsection: the output of layer l on a CompNode is its input of layer l+1, so
// the packed row order persists: only the first layer gathers and only the last one scatters.
static size_t stack_hidden_bytes(const cascade_plan *plan, const cascade_layer_desc *d) {
    return align_up((size_t)plan->batch * plan->seq_len * d->d_model * esize(d->dtype), 256);
}

extern "C" size_t cascade_layer_stack_workspace_bytes(const cascade_plan *plan, const cascade_layer_desc *d,
                                                      int32_t n_layers) {
    if (check_layer_desc(plan, d) != CASCADE_OK || n_layers <= 0) return 0;
    return layer_ws(plan, d).total + (n_layers > 1 ? 2 * stack_hidden_bytes(plan, d) : 0);
}

extern "C" int32_t cascade_layer_stack_forward(const cascade_plan *plan, const cascade_layer_desc *d,
                                               const cascade_layer_weights *weights, int32_t n_layers,
                                               const void *h_in, void *h_out, void *workspace,
                                               size_t workspace_bytes, void *stream) {
    int32_t st = check_layer_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!weights || n_layers <= 0 || !h_in || !h_out || h_in == h_out) return CASCADE_EINVAL;
    const size_t need = cascade_layer_stack_workspace_bytes(plan, d, n_layers);
    if (!workspace || workspace_bytes < need || (uintptr_t)workspace % 256) return CASCADE_EWORKSPACE;
    const size_t lw = layer_ws(plan, d).total, hb = stack_hidden_bytes(plan, d);
    char *base = (char *)workspace;
    void *pp[2] = {base + lw, base + lw + hb};                                    // packed activations between layers
    const void *src = h_in;
    for (int l = 0; l < n_layers; ++l) {
        const bool first = l == 0, last = l == n_layers - 1;
        void *dst = last ? h_out : pp[l & 1];
        st = layer_forward_impl(plan, d, weights + l, src, dst, workspace, lw, stream, nullptr, 0,
                                first ? d->io_rows : CASCADE_ROWS_PACKED, last ? d->io_rows : CASCADE_ROWS_PACKED);
        if (st != CASCADE_OK) return st;
        src = dst;
    }
    return CASCADE_OK;
}

// ---------------------------------------------------------------------------- LM head on sharded rows
static int32_t check_lm_desc(const cascade_plan *plan, const cascade_lm_head_desc *d) {
    if (!plan || !d) return CASCADE_EINVAL;
    if (!dtype_ok(d->dtype)) return CASCADE_EUNSUPPORTED;
    if (d->d_model <= 0 || d->vocab <= 0) return CASCADE_EINVAL;
    if (d->vocab % 4) return CASCADE_EUNSUPPORTED;
    if (d->norm_kind != CASCADE_NORM_LAYERNORM && d->norm_kind != CASCADE_NORM_RMSNORM) return CASCADE_EINVAL;
    if (d->rows != CASCADE_LM_ALL_ROWS && d->rows != CASCADE_LM_LAST_ROW) return CASCADE_EINVAL;
    if (!rows_ok(d->in_rows) || (d->rows == CASCADE_LM_ALL_ROWS && !rows_ok(d->out_rows))) return CASCADE_EINVAL;
    return CASCADE_OK;
}

static int64_t lm_rows(const cascade_plan *plan, const cascade_lm_head_desc *d) {
    return d->rows == CASCADE_LM_ALL_ROWS ? (int64_t)plan->batch * plan->seq_len : plan->batch;
}

extern "C" size_t cascade_lm_head_workspace_bytes(const cascade_plan *plan, const cascade_lm_head_desc *d) {
    if (check_lm_desc(plan, d) != CASCADE_OK) return 0;
    return align_up((size_t)lm_rows(plan, d) * d->d_model * esize(d->dtype), 256);
}

extern "C" int32_t cascade_lm_head(const cascade_plan *plan, const cascade_lm_head_desc *d, const void *h_in,
                                   const void *norm_gain, const void *norm_bias, const void *w_vocab, void *logits,
                                   void *workspace, size_t workspace_bytes, void *stream) {
    int32_t st = check_lm_desc(plan, d);
    if (st != CASCADE_OK) return st;
    if (!h_in || !norm_gain || !w_vocab || !logits) return CASCADE_EINVAL;
    const size_t need = cascade_lm_head_workspace_bytes(plan, d);
    if (!workspace || workspace_bytes < need || (uintptr_t)workspace % 256) return CASCADE_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int32_t M = (int32_t)lm_rows(plan, d), D = d->d_model, V = d->vocab;
    const bool all = d->rows == CASCADE_LM_ALL_ROWS;

    // closing norm: rows gathered into packed order (ALL) or the last token's row of every sequence
    NormArgs n = {};
    n.dtype = d->dtype; n.rows = M; n.D = D; n.kind = d->norm_kind; n.eps = d->norm_eps;
    n.x = h_in; n.gain = norm_gain; n.bias = norm_bias; n.y = workspace;
    if (all) {
        n.xmap = rowmap_for(plan, d->in_rows);
    } else {
        n.xmap.map = plan->last_rows_d + (d->in_rows == CASCADE_ROWS_ORIGINAL ? plan->batch : 0);
        n.xmap.seq_len = plan->batch;
    }
    n.ymap.map = nullptr; n.ymap.seq_len = n.xmap.seq_len;
    st = launch_norm(n, s);
    if (st != CASCADE_OK) return st;

    // vocabulary projection; the weight is cut into at most three row ranges so that each stays below the
    // 2 GiB a buffer descriptor can address
    GemmArgs g = {};
    g.dtype = d->dtype; g.M = M; g.N = V; g.K = D;
    g.X = workspace; g.Y = logits;
    g.ldx = D; g.ldy = V; g.ldres = V;
    g.xmap.map = nullptr; g.xmap.seq_len = 1;
    g.ymap = all ? rowmap_for(plan, d->out_rows) : g.xmap;
    g.rmap = g.xmap;
    const int64_t max_rows = ((int64_t)0x7FFF0000 / ((int64_t)D * esize(d->dtype))) & ~(int64_t)255;
    if (max_rows <= 0 || (int64_t)V > 3 * max_rows) return CASCADE_EUNSUPPORTED;
    int32_t col = 0;
    for (int i = 0; i < 3; ++i) {
        g.W[i] = (const char *)w_vocab + (size_t)col * D * esize(d->dtype);
        col = (int32_t)std::min<int64_t>(V, col + max_rows);
        g.seg_end[i] = col;
    }
    return run_gemm(g, s);
}

extern "C" int32_t cascade_greedy_token(const void *logits, int32_t dtype, int32_t rows, int32_t vocab,
                                        int32_t *token_out, void *stream) {
    if (!logits || !token_out || rows < 0 || vocab <= 0) return CASCADE_EINVAL;
    if (!dtype_ok(dtype)) return CASCADE_EUNSUPPORTED;
    return launch_argmax_rows(dtype, logits, vocab, rows, vocab, token_out, (hipStream_t)stream);
}

extern "C" int32_t cascade_layer_forward(const cascade_plan *plan, const cascade_layer_desc *d,
                                         const cascade_layer_weights *w, const void *h_in, void *h_out,
                                         void *workspace, size_t workspace_bytes, void *stream) {
    if (!d) return CASCADE_EINVAL;
    return layer_forward_impl(plan, d, w, h_in, h_out, workspace, workspace_bytes, stream, nullptr, 0, d->io_rows,
                              d->io_rows);
}

extern "C" int32_t cascade_layer_forward_staged(const cascade_plan *plan, const cascade_layer_desc *d,
                                                const cascade_layer_weights *w, const void *h_in, void *h_out,
                                                void *workspace, size_t workspace_bytes, void *stream,
                                                void *const *stage_events, int32_t n_stage_events) {
    if (!d || n_stage_events < 0 || (n_stage_events > 0 && !stage_events)) return CASCADE_EINVAL;
    return layer_forward_impl(plan, d, w, h_in, h_out, workspace, workspace_bytes, stream, stage_events,
                              n_stage_events, d->io_rows, d->io_rows);
}
