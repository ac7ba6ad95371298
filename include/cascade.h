/*
 * libcascade: one token-sharded transformer layer on one MI355X (gfx950).
 *
 * The library computes the single-layer forward pass of Cascade (Section 5,
 * Algorithm 1) with every shard resident on one GPU: per-shard linear layers
 * (Algorithm 2, the projection that closes Algorithm 4, the MLP step that closes Algorithm 1), partial
 * attention for every (query-shard, key/value-shard) pair with row maxima m and
 * subtract-max exponential sums e (Algorithm 3), and the log-sum-exp merge of
 * the partials (the merge steps of Algorithm 4).  A plan carries the sharding R of the
 * hidden rows and, optionally, a distinct sharding S of queries / keys / values
 * (cascade_plan_create_rs); cascade_plan_create sets S = R.
 *
 * Conventions
 *  - Every function returns an int32 status (CASCADE_OK = 0).  Nothing aborts,
 *    throws or prints.  After CASCADE_EHIP, cascade_last_hip_error() returns the
 *    HIP runtime code.
 *  - Pointers are DEVICE pointers unless the name ends in _host.  The library
 *    borrows them: the caller allocates and frees.  Tensor memory is never
 *    allocated here; scratch comes from the caller's workspace.  Only
 *    cascade_plan_create allocates (the index maps it owns).
 *  - All work is enqueued on the caller's HIP stream (void* = hipStream_t) and
 *    is asynchronous; there are no hidden synchronisations.
 *  - Row-major everywhere; a weight matrix is [out_features, in_features].
 *  - "Packed" row order: shards in shard-id order, rows inside a shard in
 *    ascending original token index (the concatenation rule of the
 *    Attention-Pass subsection).  perm[r] = original index of packed row r.
 *  - dtype CASCADE_BF16: tensors are bf16, accumulation and m, e, u are fp32.
 *    dtype CASCADE_F32: everything fp32.
 *  - Empty shards are legal.  A query row that sees no key of a shard gets
 *    m = -inf, e = 0, u = 0 and weight 0 in the merge.
 */
#ifndef CASCADE_H
#define CASCADE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define CASCADE_API __attribute__((visibility("default")))
#else
#define CASCADE_API
#endif

/* status codes */
#define CASCADE_OK            0
#define CASCADE_EINVAL        1   /* null pointer or negative / zero size               */
#define CASCADE_ESHAPE        2   /* dimensions inconsistent with each other / the plan */
#define CASCADE_EASSIGN       3   /* shard id outside [0, n_shards)                     */
#define CASCADE_EUNSUPPORTED  4   /* dtype / head_dim / option not built                */
#define CASCADE_EWORKSPACE    5   /* workspace missing or too small                     */
#define CASCADE_EHIP          6   /* HIP runtime error                                  */

#define CASCADE_F32   0
#define CASCADE_BF16  1

#define CASCADE_MASK_NONE    0
#define CASCADE_MASK_CAUSAL  1   /* key visible iff position[key] <= position[query]   */

#define CASCADE_ROWS_ORIGINAL  0 /* row t of a sequence is token t                     */
#define CASCADE_ROWS_PACKED    1 /* row r of a sequence is token perm[r]               */

#define CASCADE_U_UNNORMALISED 0 /* u~ = sum_s exp(a - m) v_s  (= e * u)               */
#define CASCADE_U_NORMALISED   1 /* u  = softmax(a^{S_j S_k}) v^{S_k} (Algorithm 3)    */

#define CASCADE_NORM_NONE      0
#define CASCADE_NORM_LAYERNORM 1
#define CASCADE_NORM_RMSNORM   2

#define CASCADE_ACT_GELU_ERF   0
#define CASCADE_ACT_GELU_TANH  1
#define CASCADE_ACT_SWIGLU     2

#define CASCADE_ATTN_FUSED        0 /* running merge in registers, no partials written */
#define CASCADE_ATTN_MATERIALISED 1 /* partial_attn -> m, e, u~ in HBM -> lse_merge     */

/* epilogue flags of cascade_shard_gemm (bit mask) */
#define CASCADE_EPI_BIAS       1
#define CASCADE_EPI_GELU_ERF   2
#define CASCADE_EPI_GELU_TANH  4
#define CASCADE_EPI_SWIGLU     8   /* Y = silu(X W^T) * (X W_up^T)                      */
#define CASCADE_EPI_ROPE       16  /* rotate the first rope_cols columns head by head   */
#define CASCADE_EPI_RESIDUAL   32  /* Y += residual                                     */

/* ------------------------------------------------------------------ shard plan
 * Section 5.1: the partition of [N] into shards, as index maps.  Built on the
 * host from token_to_shard_host[seq_len] (values in [0, n_shards)), copied to
 * the current device.  positions_host[seq_len] gives each token's position for
 * the causal mask and the rotary embedding (NULL: position t = t).  The same
 * assignment is shared by all `batch` sequences.
 * Errors: EINVAL (null out / host array, sizes <= 0, unknown mask kind),
 * EASSIGN (shard id out of range), EHIP.                                       */
typedef struct cascade_plan cascade_plan;

CASCADE_API int32_t cascade_plan_create(cascade_plan **out, int32_t batch, int32_t seq_len, int32_t n_shards,
                            const int32_t *token_to_shard_host, const int32_t *positions_host,
                            int32_t mask_kind);

/* Device pointers to perm[seq_len], inv_perm[seq_len], offsets[n_shards + 1]
 * (int32, owned by the plan); any out pointer may be NULL.                     */
CASCADE_API int32_t cascade_plan_maps(const cascade_plan *plan, const int32_t **perm_dev,
                          const int32_t **inv_perm_dev, const int32_t **offsets_dev);

/* Host copies of the same maps (owned by the plan).                            */
CASCADE_API int32_t cascade_plan_maps_host(const cascade_plan *plan, const int32_t **perm_host,
                               const int32_t **inv_perm_host, const int32_t **offsets_host);

/* Section 5.1 keeps the sharding of hidden states {R_i} (alpha shards) apart from
 * the sharding of queries / keys / values {S_j} (beta shards); Section 6.4 refines
 * R into S by an m-split.  This variant takes both: token_to_row_shard_host
 * defines the packed row order and the row shards (as token_to_shard_host does
 * above); token_to_kv_shard_host[seq_len] (values in [0, n_kv_shards)) defines the
 * key/value shards S_k.  Partials then have one entry per key/value shard:
 * m, e [B,H,n_kv_shards,N], u [B,n_kv_shards,H,N,d], rows in the row partition's
 * packed order; cascade_lse_merge merges over the n_kv_shards partials.  Keys of
 * S_k are taken in ascending token index (the sorted concatenation rule of the
 * Attention-Pass subsection).  The result of the merged attention does not depend
 * on either partition.  Errors as cascade_plan_create.                          */
CASCADE_API int32_t cascade_plan_create_rs(cascade_plan **out, int32_t batch, int32_t seq_len, int32_t n_row_shards,
                               const int32_t *token_to_row_shard_host, int32_t n_kv_shards,
                               const int32_t *token_to_kv_shard_host, const int32_t *positions_host,
                               int32_t mask_kind);

/* Host copies of the key/value partition's maps (owned by the plan): its shard
 * count, kv_perm[seq_len] (kv-packed row -> token), kv_offsets[n_kv_shards + 1],
 * kv_to_row[seq_len] (kv-packed row -> packed row of the row partition; NULL is
 * returned when the plan has a single partition).  Any out pointer may be NULL.  */
CASCADE_API int32_t cascade_plan_kv_maps_host(const cascade_plan *plan, int32_t *n_kv_shards,
                                  const int32_t **kv_perm_host, const int32_t **kv_offsets_host,
                                  const int32_t **kv_to_row_host);

/* (c, delta)-sharding of Section 6: 0-based token t belongs to shard
 * (t mod delta) div c; writes token_to_shard_host[seq_len] and the shard count
 * ceil(delta / c) (n_shards may be NULL).  Host only.  Errors: EINVAL.           */
CASCADE_API int32_t cascade_cdelta_assignment(int32_t seq_len, int32_t c, int32_t delta,
                                  int32_t *token_to_shard_host, int32_t *n_shards);

/* m-split of Section 6.4: the sorted tokens of row shard i are dealt round-robin
 * into m pieces (piece x takes the elements at sorted indices x, x + m, ...), and
 * piece x of shard i becomes key/value shard m i + x (0-based), so there are
 * m * n_row_shards key/value shards.  Writes token_to_kv_shard_host[seq_len].
 * Host only.  Errors: EINVAL, EASSIGN (row shard id out of range), EUNSUPPORTED. */
CASCADE_API int32_t cascade_m_split(int32_t seq_len, int32_t n_row_shards, const int32_t *token_to_row_shard_host,
                        int32_t m, int32_t *token_to_kv_shard_host);

/* Cost model of the multi-party setting the method was designed for (Equation 1
 * and the rounds count of the Communication Analysis appendix); on one GPU these
 * are the bytes MATERIALISED mode moves through HBM.  Per layer:
 *   stage_a_bytes = beta F d (H + 2 H_KV) N     q, k, v rows to the AttnNodes
 *   stage_b_bytes = beta F (d + 2) H N          m, e, u rows back
 *   rounds        = 2 alpha beta^2, or 2 beta^2 when m_split_scheme != 0
 *                   ((c, delta)-sharding with an m-split: beta = m alpha)
 * with alpha = n_row_shards, beta = n_kv_shards, F = bytes_per_value.  Any out
 * pointer may be NULL.  Host only.  Errors: EINVAL.                              */
CASCADE_API int32_t cascade_comm_cost(int32_t n_row_shards, int32_t n_kv_shards, int32_t m_split_scheme,
                          int32_t bytes_per_value, int32_t head_dim, int32_t n_heads, int32_t n_kv_heads,
                          int64_t seq_len, int64_t *stage_a_bytes, int64_t *stage_b_bytes, int64_t *rounds);

/* Equation 2 (Theoretical Costs): communication time of one layer under perfect
 * parallel transport, node bandwidth B (bytes/s) and inter-node latency tau (s):
 *   stage_a_s = tau + beta F d (H + 2 H_KV) / B * max_i |R_i|
 *   stage_b_s = tau + F (d + 2) H / B * max_j |S_j|
 *   total_s   = stage_a_s + stage_b_s
 * With a plan, beta = its key/value shard count and the two maxima are taken from its
 * partitions (n_kv_shards, max_row_shard, max_kv_shard are then ignored); with
 * plan == NULL the three are the caller's.  Out pointers are HOST doubles, any may be
 * NULL.  Host only.  Errors: EINVAL (non-positive sizes, negative or NaN latency,
 * bandwidth not above zero).                                                      */
CASCADE_API int32_t cascade_comm_time(const cascade_plan *plan, int32_t n_kv_shards, int32_t max_row_shard,
                          int32_t max_kv_shard, int32_t bytes_per_value, int32_t head_dim,
                          int32_t n_heads, int32_t n_kv_heads, double latency_s,
                          double bandwidth_bytes_per_s, double *stage_a_s, double *stage_b_s,
                          double *total_s);

CASCADE_API void cascade_plan_destroy(cascade_plan *plan);

/* Bytes of caller-owned workspace an entry point needs, by operation: desc points to
 * the descriptor type of that operation; flags is the layer count for
 * CASCADE_OP_LAYER_STACK and ignored otherwise.  Operations without a workspace
 * (shard GEMM, LSE merge, decode, norm) and invalid descriptors give 0.  The
 * per-operation queries below return the same numbers.                          */
#define CASCADE_OP_SHARD_GEMM     0   /* cascade_gemm_desc: no workspace               */
#define CASCADE_OP_PARTIAL_ATTN   1   /* cascade_attn_desc                             */
#define CASCADE_OP_LSE_MERGE      2   /* cascade_attn_desc: no workspace               */
#define CASCADE_OP_LAYER_FORWARD  3   /* cascade_layer_desc                            */
#define CASCADE_OP_LAYER_STACK    4   /* cascade_layer_desc, flags = n_layers          */
#define CASCADE_OP_LM_HEAD        5   /* cascade_lm_head_desc                          */
CASCADE_API size_t cascade_workspace_bytes(const cascade_plan *plan, const void *desc, int32_t op, int32_t flags);

/* HIP error code of the last CASCADE_EHIP on this thread (0 if none).          */
CASCADE_API int32_t cascade_last_hip_error(void);

/* ------------------------------------------------------------------ shard GEMM
 * The token-as-batch linear layers (Section 5 overview; Appendix C): for every
 * shard, Y[rows of the shard] = epilogue(X[rows of the shard] W^T).  Weights are
 * shared by all shards, so the groups are row-index lists; one launch covers
 * all shards.  rows must be batch * seq_len of the plan when any row map is
 * CASCADE_ROWS_ORIGINAL-to-packed (see x_rows / y_rows / res_rows).
 *
 * Row maps: the GEMM's own row r (0 <= r < rows) is a PACKED row.  With
 * x_rows = CASCADE_ROWS_ORIGINAL the kernel reads X row b*N + perm[r mod N]
 * (gather); with CASCADE_ROWS_PACKED it reads row r.  y_rows and res_rows do the
 * same for the store of Y (scatter) and the read of the residual.               */
typedef struct cascade_gemm_desc {
    int32_t dtype;      /* element type of X, W, W_up, bias, residual, Y             */
    int32_t rows;       /* M                                                          */
    int32_t k;          /* in_features                                                */
    int32_t n_out;      /* out_features = columns of Y                                */
    int32_t epilogue;   /* CASCADE_EPI_* mask; order: +bias, activation / swiglu,
                           rope, +residual                                            */
    int32_t x_rows;     /* CASCADE_ROWS_*                                             */
    int32_t y_rows;
    int32_t res_rows;
    int32_t rope_cols;  /* EPI_ROPE: columns [0, rope_cols) are rotated, in heads of
                           head_dim columns, half-split pairing (i, i + head_dim/2),
                           angle position * theta^(-2i/head_dim)                      */
    int32_t head_dim;
    float   rope_theta;
} cascade_gemm_desc;

/* X [rows, k]; W [n_out, k]; W_up [n_out, k] (EPI_SWIGLU only, else NULL);
 * bias [n_out] (EPI_BIAS; with SWIGLU unsupported); residual [rows, n_out];
 * Y [rows, n_out].  Y must not alias X.  Y may alias residual only when
 * y_rows == res_rows.
 * Errors: EINVAL, ESHAPE (rows != batch*seq_len with a map), EUNSUPPORTED
 * (bf16 needs k % 8 == 0; rope needs head_dim even and rope_cols % head_dim == 0).*/
CASCADE_API int32_t cascade_shard_gemm(const cascade_plan *plan, const cascade_gemm_desc *desc,
                           const void *X, const void *W, const void *W_up, const void *bias,
                           const void *residual, void *Y, void *stream);

/* ------------------------------------------------------------------ attention
 * Strides are in elements; the head_dim axis is contiguous.  A stride of 0
 * means "dense [B, heads, N, d]".                                               */
typedef struct cascade_attn_desc {
    int32_t dtype;        /* of q, k, v and of o                                      */
    int32_t n_heads;      /* H                                                        */
    int32_t n_kv_heads;   /* H_KV, divides H; query head h reads kv head h/(H/H_KV)   */
    int32_t head_dim;     /* d: bf16 path 64 or 128; f32 path any d <= 256            */
    float   scale;        /* a = scale * q k^T + s                                    */
    int32_t row_layout;   /* rows of q, k, v (partial_attn) and of o (lse_merge)      */
    int32_t u_mode;       /* CASCADE_U_*                                              */
    int64_t q_stride_b, q_stride_h, q_stride_n;
    int64_t kv_stride_b, kv_stride_h, kv_stride_n;   /* shared by k and v             */
} cascade_attn_desc;

/* Bytes of workspace cascade_partial_attn needs (0 is possible).                */
CASCADE_API size_t cascade_partial_attn_workspace_bytes(const cascade_plan *plan, const cascade_attn_desc *desc);

/* Algorithm 3 for every pair (j, k).  Outputs are fp32 and in PACKED row order:
 *   m, e [B, H, n_shards, N]   m[b,h,k,r], e[b,h,k,r]: packed query row r against shard k
 *   u    [B, n_shards, H, N, d]
 * m is in the units of a (natural-log domain).
 * Errors: EINVAL, ESHAPE (H % H_KV), EUNSUPPORTED (head_dim), EWORKSPACE.       */
CASCADE_API int32_t cascade_partial_attn(const cascade_plan *plan, const cascade_attn_desc *desc,
                             const void *q, const void *k, const void *v,
                             float *m, float *e, float *u,
                             void *workspace, size_t workspace_bytes, void *stream);

/* cascade_partial_attn for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as cascade_partial_attn
 * (bit-identical outputs: the same kernels run); the scratch memory of the bf16
 * kernels is a static device array of CASCADE_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends.  The call allocates nothing and
 * frees nothing.  A problem whose cascade_partial_attn_workspace_bytes exceeds
 * CASCADE_STATIC_SCRATCH_BYTES (36 MiB) is refused with CASCADE_EWORKSPACE.  The
 * bf16 kernels need 2 B H_KV d (N + N') bytes, N' = 64 x the number of 64-key
 * tiles of the key/value shards (N rounded up shard by shard); the limit covers
 * 8 kv heads of 128 at N = 8192 in 64-row-aligned shards.  fp32 needs none.
 * All calls on one GPU share that GPU's array: calls that overlap in time on the
 * same GPU (different streams or threads) race and must be serialised by the
 * caller.  Nothing in the array needs to start at zero; every call rewrites what
 * it reads.                                                                      */
#define CASCADE_STATIC_SCRATCH_BYTES (36u << 20)
CASCADE_API int32_t cascade_partial_attn_static(const cascade_plan *plan, const cascade_attn_desc *desc,
                                    const void *q, const void *k, const void *v,
                                    float *m, float *e, float *u, void *stream);

/* The merge of Algorithm 4 (Post-Pass): n = max_k m_k; w = sum_k exp(m_k - n) e_k;
 * o = sum_k exp(m_k - n) e_k u_k / w (u~ form: sum_k exp(m_k - n) u~_k / w).
 * o [B, N, H*d] in desc->dtype, rows per desc->row_layout; lse_out (optional,
 * may be NULL) [B, H, N] fp32 = n + log w, packed rows.                         */
CASCADE_API int32_t cascade_lse_merge(const cascade_plan *plan, const cascade_attn_desc *desc,
                          const float *m, const float *e, const float *u,
                          void *o, float *lse_out, void *stream);

/* ------------------------------------------------------------------ whole layer
 * Algorithm 1 on one GPU: h1 = h + o_proj(attention(norm1(h))),
 * h_out = h1 + FFN(norm2(h1)); pre-norm block.                                  */
/* Where the two norms of the block sit (the Pre-Pass subsection and the last step of
 * Algorithm 1 leave the block's internals to the model):
 *   PRE :  h1 = h + Attn(norm1(h));      out = h1 + MLP(norm2(h1))      (GPT / Llama)
 *   POST:  h1 = norm1(h + Attn(h));      out = norm2(h1 + MLP(h1))      (BERT, the
 *          model of the paper's timing runs; use a plan with CASCADE_MASK_NONE for
 *          its bidirectional attention)                                           */
#define CASCADE_NORM_PRE  0
#define CASCADE_NORM_POST 1

typedef struct cascade_layer_desc {
    int32_t dtype;
    int32_t d_model, n_heads, n_kv_heads, head_dim, d_ff;
    int32_t norm_kind;    /* CASCADE_NORM_LAYERNORM | CASCADE_NORM_RMSNORM            */
    float   norm_eps;
    int32_t act;          /* CASCADE_ACT_*                                            */
    int32_t rope;         /* 0: none, 1: half-split rotary on q and k                 */
    float   rope_theta;
    float   scale;
    int32_t attn_mode;    /* CASCADE_ATTN_*                                           */
    int32_t io_rows;      /* row order of h_in and h_out: CASCADE_ROWS_*              */
    int32_t norm_placement;   /* CASCADE_NORM_PRE (0) | CASCADE_NORM_POST             */
} cascade_layer_desc;

/* Device pointers, borrowed.  Matrices [out, in].  NULL = absent (biases, norm
 * biases, w_gate unless SWIGLU).                                                */
typedef struct cascade_layer_weights {
    const void *wq, *wk, *wv, *wo;          /* [H d, D] [Hkv d, D] [Hkv d, D] [D, H d] */
    const void *w_gate, *w_up, *w_down;     /* [f, D] [f, D] [D, f]                    */
    const void *bq, *bk, *bv, *bo, *b_up, *b_down;
    const void *norm1_g, *norm1_b, *norm2_g, *norm2_b;   /* [D]                        */
} cascade_layer_weights;

CASCADE_API size_t cascade_layer_workspace_bytes(const cascade_plan *plan, const cascade_layer_desc *desc);

/* h_in, h_out [B, N, D]; must not alias.
 * Errors: EINVAL, ESHAPE, EUNSUPPORTED, EWORKSPACE, EHIP.                       */
CASCADE_API int32_t cascade_layer_forward(const cascade_plan *plan, const cascade_layer_desc *desc,
                              const cascade_layer_weights *weights,
                              const void *h_in, void *h_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/* n_layers consecutive layers with the same descriptor and one weight set each
 * (weights[0 .. n_layers-1]): the output of layer l is the input of layer l+1 on
 * the same rows (Single Layer Pipeline subsection).  Only the first layer gathers
 * h_in into packed order and only the last one scatters into h_out (both in
 * desc->io_rows order); between layers the activations stay packed, in two
 * buffers taken from the workspace (cascade_layer_stack_workspace_bytes).
 * h_in, h_out [B, N, D]; must not alias.  Errors as cascade_layer_forward.       */
CASCADE_API size_t cascade_layer_stack_workspace_bytes(const cascade_plan *plan, const cascade_layer_desc *desc,
                                           int32_t n_layers);
CASCADE_API int32_t cascade_layer_stack_forward(const cascade_plan *plan, const cascade_layer_desc *desc,
                                    const cascade_layer_weights *weights, int32_t n_layers,
                                    const void *h_in, void *h_out,
                                    void *workspace, size_t workspace_bytes, void *stream);

/* ---- LM head on sharded rows -------------------------------------------------
 * After the last layer every CompNode applies the LM head to its own hidden rows
 * and holds R_i-sharded logits; the CompNode that holds the last token turns its
 * logits row into the next token (Single Layer Pipeline subsection, the
 * paragraph after Algorithm 1).  logits = W_vocab . norm_f(h): the model's
 * closing normalisation, then the vocabulary projection as one shard GEMM over
 * the packed rows (weights shared by all shards).
 *
 * rows = CASCADE_LM_ALL_ROWS: logits [B, N, vocab] for every token, h_in rows in
 *   in_rows order, logits rows in out_rows order (CASCADE_ROWS_*).
 * rows = CASCADE_LM_LAST_ROW: logits [B, vocab] of the token with the largest
 *   position in each sequence (lowest index among equal positions); out_rows is
 *   ignored.
 * h_in [B, N, D], norm_gain [D], norm_bias [D] or NULL, w_vocab [vocab, D],
 * logits in desc->dtype: device pointers, borrowed.  workspace: device,
 * 256-byte aligned, cascade_lm_head_workspace_bytes (the normalised rows).
 * vocab % 4 == 0.  Errors: EINVAL, ESHAPE, EUNSUPPORTED, EWORKSPACE, EHIP.       */
#define CASCADE_LM_ALL_ROWS 0
#define CASCADE_LM_LAST_ROW 1

typedef struct cascade_lm_head_desc {
    int32_t dtype;
    int32_t d_model, vocab;
    int32_t norm_kind;    /* CASCADE_NORM_LAYERNORM | CASCADE_NORM_RMSNORM            */
    float   norm_eps;
    int32_t rows;         /* CASCADE_LM_ALL_ROWS | CASCADE_LM_LAST_ROW                */
    int32_t in_rows;      /* row order of h_in: CASCADE_ROWS_*                        */
    int32_t out_rows;     /* row order of the logits (ALL_ROWS): CASCADE_ROWS_*       */
} cascade_lm_head_desc;

CASCADE_API size_t cascade_lm_head_workspace_bytes(const cascade_plan *plan, const cascade_lm_head_desc *desc);
CASCADE_API int32_t cascade_lm_head(const cascade_plan *plan, const cascade_lm_head_desc *desc,
                        const void *h_in, const void *norm_gain, const void *norm_bias,
                        const void *w_vocab, void *logits,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Greedy choice: token_out[r] (device int32 [rows]) = lowest index of the
 * largest of logits[r, 0 .. vocab) (device, [rows, vocab] in dtype).  NaNs never
 * win; a row of NaNs gives 0.  Errors: EINVAL, EUNSUPPORTED, EHIP.               */
CASCADE_API int32_t cascade_greedy_token(const void *logits, int32_t dtype, int32_t rows, int32_t vocab,
                             int32_t *token_out, void *stream);

/* The same computation with stage boundaries marked for measurement: HIP event
 * stage_events[i] (hipEvent_t, created by the caller, NULL entries skipped) is
 * recorded on the stream at boundary i.  Boundaries (CASCADE_N_STAGE_EVENTS):
 * 0 start, 1 gather+norm1, 2 qkv GEMM, 3 rotary (same instant as 2 when the
 * rotation ran in the GEMM's epilogue: bf16 pre-norm layers), 4 attention (partial
 * attention), 5 LSE merge (same instant as 4 in FUSED mode), 6 o projection +
 * residual, 7 norm2, 8 FFN up/gate GEMM, 9 FFN down + residual + scatter.       */
#define CASCADE_N_STAGE_EVENTS 10
CASCADE_API int32_t cascade_layer_forward_staged(const cascade_plan *plan, const cascade_layer_desc *desc,
                                     const cascade_layer_weights *weights,
                                     const void *h_in, void *h_out,
                                     void *workspace, size_t workspace_bytes, void *stream,
                                     void *const *stage_events, int32_t n_stage_events);

/* After a MATERIALISED cascade_layer_forward: device pointers into the workspace
 * it used, holding m, e [B,H,n_shards,N] and u~ [B,n_shards,H,N,d] (fp32).      */
CASCADE_API int32_t cascade_layer_partials(const cascade_plan *plan, const cascade_layer_desc *desc,
                               void *workspace, float **m, float **e, float **u);

/* After a cascade_layer_forward (either attention mode): device pointer into the
 * workspace it used, to the merged attention output o [B * N, H * d] in desc->dtype,
 * PACKED rows (the input of the o projection; Algorithm 4 before its last step).
 * Exposed so that the fused path can be checked at the same point as
 * cascade_lse_merge's output.  Errors: EINVAL, EUNSUPPORTED.                     */
CASCADE_API int32_t cascade_layer_attention_output(const cascade_plan *plan, const cascade_layer_desc *desc,
                                       void *workspace, void **o);

/* ------------------------------------------------------------------ KV-cache decode
 * Cost Optimizations appendix ("Caching"): in single-token generation only the
 * newest token's query row is attended, by AttnNode_jk for every kv shard k,
 * against the keys and values of S_k cached so far (the new token's own k, v
 * already appended to its shard by the caller).  One partial per shard:
 *   m, e [B, H, n_shards]        (= [B, H, n_shards, 1] of cascade_partial_attn)
 *   u    [B, n_shards, H, d]     fp32, CASCADE_U_* as in desc->u_mode
 * which cascade_lse_merge combines when called with a plan of seq_len 1 and the
 * same n_shards (cascade_plan_create(batch, 1, n_shards, {j}, ...)).
 *   q [B, H, d]; k_cache, v_cache [B, H_KV, n_shards, shard_capacity, d] (dense,
 *   desc->dtype, 16-byte aligned); shard_len_dev [B, n_shards] int32 DEVICE:
 *   rows of each shard that are valid (clamped to shard_capacity; 0 gives
 *   m = -inf, e = 0, u = 0).  No mask: every cached key is at or before the new
 *   position.  From desc: dtype, n_heads, n_kv_heads, head_dim, scale, u_mode
 *   (row_layout and strides are ignored).  head_dim must be 8 * 2^j (bf16) or
 *   4 * 2^j (f32), at most 512 / 256.
 * Errors: EINVAL, ESHAPE (H % H_KV), EUNSUPPORTED (head_dim, alignment), EHIP.   */
CASCADE_API int32_t cascade_decode_partial_attn(const cascade_attn_desc *desc, int32_t batch, int32_t n_shards,
                                    int32_t shard_capacity, const int32_t *shard_len_dev,
                                    const void *q, const void *k_cache, const void *v_cache,
                                    float *m, float *e, float *u, void *stream);

/* Normalisation of `rows` rows of D values (the optional normalisation step of
 * the Pre-Pass subsection, exposed for callers that compose a
 * single-token step themselves): y = norm(x) * gain (+ bias), statistics in
 * fp32.  x, y [rows, D], gain [D], bias [D] or NULL: device, dtype; x == y allowed.
 * Errors: EINVAL, EUNSUPPORTED, EHIP.                                            */
CASCADE_API int32_t cascade_norm(int32_t dtype, int32_t rows, int32_t d_model, int32_t norm_kind, float eps,
                     const void *x, const void *gain, const void *bias, void *y, void *stream);

/* Token-sharded KV cache from a prefill ("Caching": every AttnNode_jk keeps the
 * k, v of its shard S_k between tokens).  Copies the keys (rotary embedding
 * already applied) and values that the last cascade_layer_forward /
 * cascade_layer_stack_forward call with this plan and descriptor left in
 * `workspace` into the slabs cascade_decode_partial_attn reads:
 *   k_cache, v_cache [B, H_KV, n_kv_shards, shard_capacity, d] in desc->dtype;
 *   row r of kv shard k (ascending token index inside the shard) goes to slab
 *   row r; slab rows past the shard's size are left untouched.
 *   shard_len_dev [B, n_kv_shards] int32 DEVICE receives the shard sizes.
 * shard_capacity must hold the largest shard (ESHAPE otherwise).  The workspace
 * must not have been reused since that forward call.
 * Errors: EINVAL, ESHAPE, EUNSUPPORTED, EHIP.                                    */
CASCADE_API int32_t cascade_layer_kv_to_cache(const cascade_plan *plan, const cascade_layer_desc *desc,
                                  const void *workspace, void *k_cache, void *v_cache,
                                  int32_t shard_capacity, int32_t *shard_len_dev, void *stream);

/* ------------------------------------------------------------------ measured ceiling
 * Not a step of the method: the rate (TFLOP/s) this device sustains on back-to-back
 * bf16 16x16x32 MFMAs with random operands, for the roofline figures quoted next
 * to the datasheet peak.  lds_operands = 0: operands stay in registers;
 * 1: operands are re-read from LDS at the shard GEMM's ratio (12 16-byte reads per
 * 32 MFMAs).  One workgroup of 8 wavefronts per compute unit, `iters` (1..2^22)
 * iterations of 32 MFMAs each; runs twice on `stream`, synchronises, and reports
 * the second run.  tflops_out is a HOST pointer.  Allocates 256 bytes of device
 * memory for the duration of the call.  Errors: EINVAL, EHIP.                    */
CASCADE_API int32_t cascade_mfma_ceiling(int32_t lds_operands, int32_t iters, float *tflops_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_H */
