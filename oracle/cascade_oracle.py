"""Float64 CPU oracle for one token-sharded transformer layer (Cascade, Section 5).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
library is checked against.  It shares no code with the HIP path, is never
imported by the product package, and may be used only from tests/, the smoke
check and the benchmark's cpu_baseline leg.

Two independent routes to the same result are written out:

* layer_direct   -- the ordinary, unsharded pre-norm transformer layer.  Section 5
                    (the exactness statement after the method's introduction, and
                    the merge derivation of the Post-Pass subsection) says the
                    sharded pipeline reproduces exactly this, so it is the
                    definition of the result.
* layer_sharded  -- Algorithm 1 step by step: Algorithm 2 (pre-pass) on every hidden
                    shard, Algorithm 3 (attention-pass) on every (query-shard,
                    key/value-shard) pair, Algorithm 4 (post-pass) on every hidden
                    shard, then the residual and MLP.

All arithmetic is float64 numpy; matmul (@) is the only library contraction used.

Readings taken where the paper is silent or inconsistent (each is also listed in
the design notes):
  * a = scale * q k^T + s with an explicit scale (the paper prints none; scale=1
    gives its formula literally, 1/sqrt(d) gives the standard layer).
  * A query row that sees no key of S_k has m = -inf, e = 0, u = 0 and weight 0 in
    the merge; exp(-inf - (-inf)) is never evaluated.
  * The post-pass maximum n depends on the row only (the maximum step of Algorithm 4), not on k.
  * u has shape (H, rows, d) (Appendix D), not (H, N, |S_k|) as Table 2 prints.
  * mlp(h + o) is the rest of a pre-norm block: h1 = h + o, out = h1 + FFN(norm2(h1)).
  * The causal mask compares original token positions: s[x, y] = 0 if pos[y] <= pos[x]
    else -inf; it is the same for every head.
  * Rows inside a shard are in ascending original index (Attention-Pass subsection).
  * Query head h reads key/value head h // (H / H_KV) (repeat_kv of Algorithm 3).
  * R = S (the option named at the start of the AttnNode security subsection).
"""
import numpy as np
from scipy.special import erf

F64 = np.float64


# --------------------------------------------------------------------------- sharding
def shard_index_lists(token_to_shard, n_shards):
    """Section 5.1: the partition {S_j}; each list ascending (Attention-Pass subsection)."""
    a = np.asarray(token_to_shard)
    if a.ndim != 1 or (a.size and (a.min() < 0 or a.max() >= n_shards)):
        raise ValueError("token_to_shard must be 1-D with values in [0, n_shards)")
    return [np.flatnonzero(a == j) for j in range(n_shards)]


def shard_plan(token_to_shard, n_shards):
    """Packed order: shards in shard-id order, rows ascending inside a shard.

    Returns offsets[n_shards+1], perm[N] (packed row -> original index) and
    inv_perm[N] (original index -> packed row).
    """
    lists = shard_index_lists(token_to_shard, n_shards)
    sizes = np.array([len(x) for x in lists], dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    perm = (np.concatenate(lists) if lists else np.zeros(0)).astype(np.int32)
    inv_perm = np.empty_like(perm)
    inv_perm[perm] = np.arange(perm.size, dtype=np.int32)
    return offsets, perm, inv_perm


def cdelta_assignment(seq_len, c, delta):
    """(c, delta)-sharding (Definition in Section 6): 0-based token t belongs to the
    shard (t mod delta) div c; alpha = ceil(delta / c) shards."""
    t = np.arange(seq_len)
    return ((t % delta) // c).astype(np.int32)


def m_split(index_list, m):
    """m-split of a sorted hidden shard R_i into R_{i,1..m} (AttnNode security
    subsection).  The worked N=18 example takes every m-th element of sorted R_i
    starting at x, which is what is done here (the prose's stride 'delta' is in
    token positions, not list indices, when m = c)."""
    r = np.sort(np.asarray(index_list))
    return [r[x::m] for x in range(m)]


def m_split_assignment(token_to_row_shard, n_row_shards, m):
    """The S sharding formed from an R sharding by the m-split (AttnNode Full Security
    subsection): beta = m alpha and S_{m(i-1)+x} = R_{i,x} (1-based), i.e. 0-based kv
    shard m*i + x holds piece x of row shard i.  Returns token_to_kv_shard."""
    out = np.empty(len(token_to_row_shard), dtype=np.int32)
    for i, R in enumerate(shard_index_lists(token_to_row_shard, n_row_shards)):
        for x, piece in enumerate(m_split(R, m)):
            out[piece] = m * i + x
    return out


# --------------------------------------------------------------------------- per-token pieces
def layer_norm(x, gain, bias, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps) * gain
    return y + bias if bias is not None else y


def rms_norm(x, gain, eps):
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def norm(x, kind, gain, bias, eps):
    if kind == "layernorm":
        return layer_norm(x, gain, bias, eps)
    if kind == "rmsnorm":
        return rms_norm(x, gain, eps)
    raise ValueError(kind)


def gelu_erf(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def linear(x, w, b=None):
    y = x @ w.T
    return y + b if b is not None else y


def rope(x, pos, theta):
    """Rotary embedding, half-split pairing: element i pairs with i + d/2 and is
    rotated by pos * theta**(-2i/d).  x is (..., rows, d); pos is (rows,), the
    ORIGINAL token positions of those rows (Pre-Pass subsection: p^{R_i} depends
    only on the index set R_i)."""
    d = x.shape[-1]
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=F64) / d)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def ffn(x, w, act):
    if act == "swiglu":
        return linear(silu(linear(x, w["w_gate"])) * linear(x, w["w_up"]), w["w_down"])
    g = gelu_erf if act == "gelu" else gelu_tanh
    return linear(g(linear(x, w["w_up"], w.get("b_up"))), w["w_down"], w.get("b_down"))


def mask_block(pos_q, pos_k, mask_kind):
    """Additive mask s[x, y] for query positions pos_q and key positions pos_k."""
    if mask_kind == "none":
        return np.zeros((len(pos_q), len(pos_k)), dtype=F64)
    vis = np.asarray(pos_k)[None, :] <= np.asarray(pos_q)[:, None]
    return np.where(vis, 0.0, -np.inf)


def _f64_weights(w):
    return {k: np.asarray(v, dtype=F64) for k, v in w.items()}


def _split_heads(x, n_heads, d):
    # (rows, n_heads*d) -> (n_heads, rows, d)
    return x.reshape(x.shape[0], n_heads, d).transpose(1, 0, 2)


# --------------------------------------------------------------------------- Algorithm 2
def pre_pass(h_rows, pos_rows, w, cfg):
    """Algorithm 2 on one hidden shard: norm (absent in a post-norm block), q/k/v
    projection, rotary embedding."""
    post = getattr(cfg, "norm_placement", "pre") == "post"
    x = h_rows if post else norm(h_rows, cfg.norm, w["norm1_g"], w.get("norm1_b"), cfg.eps)
    q = _split_heads(linear(x, w["wq"], w.get("bq")), cfg.n_heads, cfg.head_dim)
    k = _split_heads(linear(x, w["wk"], w.get("bk")), cfg.n_kv_heads, cfg.head_dim)
    v = _split_heads(linear(x, w["wv"], w.get("bv")), cfg.n_kv_heads, cfg.head_dim)
    if cfg.rope:
        q = rope(q, pos_rows, cfg.rope_theta)
        k = rope(k, pos_rows, cfg.rope_theta)
    return q, k, v


# --------------------------------------------------------------------------- Algorithm 3
def attn_pass(q, k, v, s, scale=1.0):
    """The three quantities an AttnNode returns for one (query-shard, key/value-shard) pair, written from their
    definitions in the Post-Pass subsection (Algorithm 3 computes the same): for query row x of head h, with
    scores a[x, y] = scale <q[h, x], k[g, y]> + s[x, y] over the keys y of the shard and g the key/value head
    that h reads,
        m[h, x] = max_y a[x, y],   e[h, x] = sum_y exp(a[x, y] - m[h, x]),
        u[h, x] = sum_y exp(a[x, y] - m[h, x]) v[g, y] / e[h, x].

    q (H, nq, d); k, v (H_KV, nk, d); s (nq, nk) additive mask.
    Returns m (H, nq), e (H, nq), u (H, nq, d); a row that sees no key has m = -inf, e = 0, u = 0.
    """
    H, nq, d = q.shape
    Hkv, nk, _ = k.shape
    m = np.full((H, nq), -np.inf)
    e = np.zeros((H, nq))
    u = np.zeros((H, nq, d))
    if nk == 0:
        return m, e, u
    heads_per_kv = H // Hkv
    for h in range(H):
        g = h // heads_per_kv
        a = scale * (q[h] @ k[g].T) + s                    # (nq, nk)
        m[h] = a.max(axis=1)
        seen = np.isfinite(m[h])                           # rows with at least one visible key
        p = np.exp(a[seen] - m[h][seen, None])
        e[h][seen] = p.sum(axis=1)
        u[h][seen] = (p @ v[g]) / e[h][seen, None]
    return m, e, u


# --------------------------------------------------------------------------- Algorithm 4 (merge)
def post_pass_merge(ms, es, us):
    """The output rows of one query shard from its beta partials, by the identity the Post-Pass subsection
    derives (the merge steps of Algorithm 4 evaluate it): with n = max_k m_k and weights
    c_k = exp(m_k - n) e_k,
        o = sum_k c_k u_k / sum_k c_k.
    A partial with m_k = -inf (no visible key in S_k) has weight 0.

    ms, es: sequences of (H, rows); us: sequence of (H, rows, d), normalised u.  Returns o (H, rows, d).
    """
    M, E, U = np.stack(ms), np.stack(es), np.stack(us)      # (beta, H, rows[, d])
    n = M.max(axis=0)
    c = np.zeros_like(M)
    live = np.isfinite(M)
    c[live] = np.exp((M - np.where(np.isfinite(n), n, 0.0))[live]) * E[live]
    total = c.sum(axis=0)
    o = (c[..., None] * U).sum(axis=0)
    return o / np.where(total > 0.0, total, 1.0)[..., None]


# --------------------------------------------------------------------------- all pairs on given q, k, v
def partial_attention_all_pairs(q, k, v, token_to_shard, n_shards, positions=None,
                                scale=1.0, mask_kind="causal"):
    """Algorithm 3 on every (j, k) pair for one sequence.

    q (H, N, d), k, v (H_KV, N, d) in ORIGINAL token order.  Outputs are in packed
    row order: m, e (H, beta, N) indexed [head, kv-shard, packed query row];
    u (beta, H, N, d) normalised.
    """
    q, k, v = (np.asarray(t, dtype=F64) for t in (q, k, v))
    H, N, d = q.shape
    pos = np.arange(N) if positions is None else np.asarray(positions)
    lists = shard_index_lists(token_to_shard, n_shards)
    offsets, _, _ = shard_plan(token_to_shard, n_shards)
    m = np.full((H, n_shards, N), -np.inf)
    e = np.zeros((H, n_shards, N))
    u = np.zeros((n_shards, H, N, d))
    for j, Sj in enumerate(lists):
        r0, r1 = offsets[j], offsets[j + 1]
        for kk, Sk in enumerate(lists):
            s = mask_block(pos[Sj], pos[Sk], mask_kind)
            mj, ej, uj = attn_pass(q[:, Sj], k[:, Sk], v[:, Sk], s, scale)
            m[:, kk, r0:r1], e[:, kk, r0:r1], u[kk, :, r0:r1] = mj, ej, uj
    return m, e, u


def partial_attention_rs(q, k, v, token_to_row_shard, n_row_shards, token_to_kv_shard, n_kv_shards,
                         positions=None, scale=1.0, mask_kind="causal"):
    """Algorithm 3 on every pair (S_j, S_k) of the query / key-value sharding S when it
    differs from the hidden-state sharding R (Section 5.1).  The rows AttnNode_jk returns
    are routed back to the CompNode that owns them (R_i ∩ S_j, Post-Pass subsection), so
    the outputs are laid out in R's packed row order:
    m, e (H, beta, N) indexed [head, kv-shard of S, R-packed query row]; u (beta, H, N, d)."""
    q, k, v = (np.asarray(t, dtype=F64) for t in (q, k, v))
    H, N, d = q.shape
    pos = np.arange(N) if positions is None else np.asarray(positions)
    s_lists = shard_index_lists(token_to_kv_shard, n_kv_shards)
    _, _, inv_perm_r = shard_plan(token_to_row_shard, n_row_shards)
    m = np.full((H, n_kv_shards, N), -np.inf)
    e = np.zeros((H, n_kv_shards, N))
    u = np.zeros((n_kv_shards, H, N, d))
    for Sj in s_lists:
        rows = inv_perm_r[Sj]                          # where CompNodes keep the rows of S_j
        for kk, Sk in enumerate(s_lists):
            s = mask_block(pos[Sj], pos[Sk], mask_kind)
            mj, ej, uj = attn_pass(q[:, Sj], k[:, Sk], v[:, Sk], s, scale)
            m[:, kk, rows], e[:, kk, rows], u[kk][:, rows] = mj, ej, uj
    return m, e, u


def lse_merge_all(m, e, u):
    """The merge steps of Algorithm 4 over the kv-shard axis of packed partials.
    m, e (H, beta, N); u (beta, H, N, d) normalised.  Returns o (N, H*d), packed rows."""
    beta = m.shape[1]
    o = post_pass_merge([m[:, kk] for kk in range(beta)], [e[:, kk] for kk in range(beta)],
                        [u[kk] for kk in range(beta)])
    H, N, d = o.shape
    return o.transpose(1, 0, 2).reshape(N, H * d)


# --------------------------------------------------------------------------- token-sharded KV-cache decode
def decode_partials(q_new, k_shards, v_shards, scale=1.0):
    """Single-token generation with cached keys and values (Cost Optimizations appendix,
    'Caching'): only the newest token's query row is attended, by AttnNode_jk for every kv
    shard k, against the rows of S_k cached so far (the new token's own key and value already
    appended to its shard).  Every cached key is at or before the new position, so the mask
    block is all zeros.  q_new (H, d); k_shards, v_shards: one (H_KV, L_k, d) array per shard
    (L_k = 0 allowed).  Returns m, e (H, beta) and u (beta, H, d), u normalised."""
    q = np.asarray(q_new, dtype=F64)[:, None, :]
    H, _, d = q.shape
    beta = len(k_shards)
    m = np.full((H, beta), -np.inf)
    e = np.zeros((H, beta))
    u = np.zeros((beta, H, d))
    for kk in range(beta):
        K, V = np.asarray(k_shards[kk], dtype=F64), np.asarray(v_shards[kk], dtype=F64)
        mk, ek, uk = attn_pass(q, K, V, np.zeros((1, K.shape[1])), scale)
        m[:, kk], e[:, kk], u[kk] = mk[:, 0], ek[:, 0], uk[:, 0]
    return m, e, u


def decode_merge(m, e, u):
    """The merge steps of Algorithm 4 for the one new row: m, e (H, beta); u (beta, H, d).  Returns o (H*d)."""
    beta = m.shape[1]
    o = post_pass_merge([m[:, kk:kk + 1] for kk in range(beta)], [e[:, kk:kk + 1] for kk in range(beta)],
                        [u[kk][:, None, :] for kk in range(beta)])
    return o[:, 0].reshape(-1)


# --------------------------------------------------------------------------- the two layer routes
def layer_direct(h, w, cfg, positions=None, mask_kind="causal", scale=None, rows=None):
    """The unsharded layer, one sequence h (N, D).  With rows given, only those
    output rows are computed (keys and values still come from every token)."""
    w = _f64_weights(w)
    h = np.asarray(h, dtype=F64)
    N = h.shape[0]
    pos = np.arange(N) if positions is None else np.asarray(positions)
    scale = cfg.scale if scale is None else scale
    rows = np.arange(N) if rows is None else np.asarray(rows)
    H, Hkv, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim

    post = getattr(cfg, "norm_placement", "pre") == "post"
    x = h if post else norm(h, cfg.norm, w["norm1_g"], w.get("norm1_b"), cfg.eps)
    k = _split_heads(linear(x, w["wk"], w.get("bk")), Hkv, d)
    v = _split_heads(linear(x, w["wv"], w.get("bv")), Hkv, d)
    q = _split_heads(linear(x[rows], w["wq"], w.get("bq")), H, d)
    if cfg.rope:
        q = rope(q, pos[rows], cfg.rope_theta)
        k = rope(k, pos, cfg.rope_theta)
    s = mask_block(pos[rows], pos, mask_kind)
    o = np.empty((len(rows), H * d))
    rep = H // Hkv
    for hh in range(H):
        a = scale * (q[hh] @ k[hh // rep].T) + s
        a = a - a.max(axis=-1, keepdims=True)
        p = np.exp(a)
        p = p / p.sum(axis=-1, keepdims=True)
        o[:, hh * d:(hh + 1) * d] = p @ v[hh // rep]
    return _block_tail(h[rows], o, w, cfg)


def _block_tail(h_rows, o, w, cfg):
    """What follows the attention values on a set of rows (the projection that closes Algorithm 4 and the last step of Algorithm 1):
    output projection, residual and MLP, with the norms before the sub-blocks ("pre", the default
    reading) or after the residual sums ("post", the BERT-shaped block of the paper's timing runs)."""
    if getattr(cfg, "norm_placement", "pre") == "post":
        h1 = norm(h_rows + linear(o, w["wo"], w.get("bo")), cfg.norm, w["norm1_g"], w.get("norm1_b"), cfg.eps)
        return norm(h1 + ffn(h1, w, cfg.act), cfg.norm, w["norm2_g"], w.get("norm2_b"), cfg.eps)
    h1 = h_rows + linear(o, w["wo"], w.get("bo"))
    x2 = norm(h1, cfg.norm, w["norm2_g"], w.get("norm2_b"), cfg.eps)
    return h1 + ffn(x2, w, cfg.act)


def layer_sharded(h, w, cfg, token_to_shard, n_shards, positions=None, mask_kind="causal",
                  scale=None, return_partials=False):
    """Algorithm 1 for one sequence h (N, D); output in original token order."""
    w = _f64_weights(w)
    h = np.asarray(h, dtype=F64)
    N = h.shape[0]
    pos = np.arange(N) if positions is None else np.asarray(positions)
    scale = cfg.scale if scale is None else scale
    lists = shard_index_lists(token_to_shard, n_shards)

    # pre-pass on every hidden shard (Algorithm 1, pre-pass step)
    qkv = [pre_pass(h[R], pos[R], w, cfg) for R in lists]

    # attention-pass on every pair (Algorithm 1, attention-pass step); with R = S the stage-A routing
    # of Algorithm 1 hands AttnNode_jk the whole of shard j's q and shard k's k, v.
    partial = {}
    for j, Sj in enumerate(lists):
        for kk, Sk in enumerate(lists):
            s = mask_block(pos[Sj], pos[Sk], mask_kind)
            partial[(j, kk)] = attn_pass(qkv[j][0], qkv[kk][1], qkv[kk][2], s, scale)

    # post-pass, residual and MLP on every hidden shard (Algorithm 1, closing steps)
    out = np.empty_like(h)
    for i, R in enumerate(lists):
        if len(R) == 0:
            continue
        ms = [partial[(i, kk)][0] for kk in range(n_shards)]
        es = [partial[(i, kk)][1] for kk in range(n_shards)]
        us = [partial[(i, kk)][2] for kk in range(n_shards)]
        o = post_pass_merge(ms, es, us)                               # Algorithm 4 merge
        o = o.transpose(1, 0, 2).reshape(len(R), -1)
        out[R] = _block_tail(h[R], o, w, cfg)                         # o projection, residual, MLP
    if return_partials:
        return out, partial
    return out


def layer_sharded_rs(h, w, cfg, token_to_row_shard, n_row_shards, token_to_kv_shard, n_kv_shards,
                     positions=None, mask_kind="causal", scale=None):
    """Algorithm 1 with distinct shardings: CompNode_i holds the hidden rows R_i, AttnNode_jk
    works on (S_j, S_k).  Output in original token order."""
    w = _f64_weights(w)
    h = np.asarray(h, dtype=F64)
    N = h.shape[0]
    pos = np.arange(N) if positions is None else np.asarray(positions)
    scale = cfg.scale if scale is None else scale
    r_lists = shard_index_lists(token_to_row_shard, n_row_shards)
    s_lists = shard_index_lists(token_to_kv_shard, n_kv_shards)
    H, Hkv, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim

    # pre-pass on every hidden shard, then stage-A routing: AttnNode_jk receives the rows
    # R_i ∩ S_j of q and R_i ∩ S_k of k, v from every CompNode_i and concatenates them in
    # sorted order (Algorithm 1, pre-pass and stage-A routing); held here as full-length arrays indexed by token
    q = np.empty((H, N, d)); k = np.empty((Hkv, N, d)); v = np.empty((Hkv, N, d))
    for R in r_lists:
        if len(R):
            q[:, R], k[:, R], v[:, R] = pre_pass(h[R], pos[R], w, cfg)

    # attention-pass on every pair of S shards (Algorithm 1, attention-pass step); stage-B routing sends row t of
    # AttnNode_jk's result to the CompNode that holds t
    m = np.full((n_kv_shards, H, N), -np.inf); e = np.zeros((n_kv_shards, H, N)); u = np.zeros((n_kv_shards, H, N, d))
    for Sj in s_lists:
        for kk, Sk in enumerate(s_lists):
            s = mask_block(pos[Sj], pos[Sk], mask_kind)
            m[kk][:, Sj], e[kk][:, Sj], u[kk][:, Sj] = attn_pass(q[:, Sj], k[:, Sk], v[:, Sk], s, scale)

    # post-pass, residual and MLP on every hidden shard (Algorithm 1, closing steps)
    out = np.empty_like(h)
    for R in r_lists:
        if len(R) == 0:
            continue
        o = post_pass_merge([m[kk][:, R] for kk in range(n_kv_shards)], [e[kk][:, R] for kk in range(n_kv_shards)],
                            [u[kk][:, R] for kk in range(n_kv_shards)])
        o = o.transpose(1, 0, 2).reshape(len(R), -1)
        out[R] = _block_tail(h[R], o, w, cfg)
    return out


def layer_stack_direct(h, layer_weights, cfg, **kw):
    """Consecutive layers (Single Layer Pipeline subsection: the output of layer l is the input of
    layer l+1 on the same CompNode); one weight dict per layer."""
    for w in layer_weights:
        h = layer_direct(h, w, cfg, **kw)
    return h


def layer_stack_sharded(h, layer_weights, cfg, token_to_shard, n_shards, **kw):
    for w in layer_weights:
        h = layer_sharded(h, w, cfg, token_to_shard, n_shards, **kw)
    return h


# --------------------------------------------------------------------------- LM head on sharded rows
def lm_head_direct(h, head, cfg):
    """Definition of the result: logits[t] = W_vocab . norm_f(h[t]) for every token t (the closing
    normalisation of the model, then the vocabulary projection).  h (N, D) -> (N, V)."""
    h = np.asarray(h, dtype=F64)
    x = norm(h, cfg.norm, np.asarray(head["norm_g"], F64),
             None if head.get("norm_b") is None else np.asarray(head["norm_b"], F64), cfg.eps)
    return linear(x, np.asarray(head["w_vocab"], F64), None)


def lm_head_sharded(h, head, cfg, token_to_shard, n_shards):
    """Single Layer Pipeline subsection, after the last layer: every CompNode_i applies the LM head to
    its own rows R_i and obtains R_i-sharded logits; they are laid back at the token positions."""
    h = np.asarray(h, dtype=F64)
    lists = shard_index_lists(token_to_shard, n_shards)
    V = np.asarray(head["w_vocab"]).shape[0]
    logits = np.empty((h.shape[0], V), dtype=F64)
    for R in lists:
        if len(R):
            logits[R] = lm_head_direct(h[R], head, cfg)
    return logits


def next_token(h, head, cfg, token_to_shard, n_shards, positions=None):
    """The CompNode that holds the last token (largest position) turns its logits row into the next
    token: greedy choice, lowest index on ties.  Returns (token id, shard that produced it, logits row)."""
    N = np.asarray(h).shape[0]
    pos = np.arange(N) if positions is None else np.asarray(positions)
    t_last = int(np.argmax(pos))
    shard = int(np.asarray(token_to_shard)[t_last])
    row = lm_head_direct(np.asarray(h, F64)[t_last:t_last + 1], head, cfg)[0]
    return int(np.argmax(row)), shard, row


def layer_direct_batch(h, w, cfg, **kw):
    return np.stack([layer_direct(h[b], w, cfg, **kw) for b in range(h.shape[0])])


def layer_sharded_batch(h, w, cfg, token_to_shard, n_shards, **kw):
    return np.stack([layer_sharded(h[b], w, cfg, token_to_shard, n_shards, **kw)
                     for b in range(h.shape[0])])


# --------------------------------------------------------------------------- cost model
def comm_bytes(beta, F, d, H, Hkv, N):
    """Equation 1 and its two halves (Appendix D): stage A ships q, k, v rows to the
    AttnNodes, stage B ships m, e, u rows back."""
    stage_a = beta * F * d * (H + 2 * Hkv) * N
    stage_b = beta * F * (d + 2) * H * N
    return stage_a + stage_b, stage_a, stage_b


def comm_time(row_lists, kv_lists, F, d, H, Hkv, tau, bandwidth):
    """Equation 2 from its derivation (Communication Analysis appendix), node by node: with perfect
    parallel transport each stage lasts one latency plus the time of the node that sends most.
    Stage A: CompNode_i sends every one of its |R_i| rows of q (H d values) and of k, v (2 H_KV d
    values) to beta AttnNodes.  Stage B: AttnNode_jk sends the |S_j| rows of u (H d values) and of m, e
    (2 H values) it computed.  row_lists / kv_lists: the index lists of {R_i} and {S_j}.
    Returns (total seconds, stage A seconds, stage B seconds)."""
    beta = len(kv_lists)
    sent_a = [beta * len(R) * (H * d + 2 * Hkv * d) * F for R in row_lists]        # bytes leaving CompNode_i
    sent_b = [len(kv_lists[j]) * (H * d + 2 * H) * F for j in range(beta) for _k in range(beta)]   # AttnNode_jk
    t_a = tau + max(sent_a) / bandwidth
    t_b = tau + max(sent_b) / bandwidth
    return t_a + t_b, t_a, t_b


def overhead_ops(H, N, d):
    """Appendix C: extra operations over the vanilla pass: (a) merge ~ H N d, (b) expsums ~ H N^2."""
    return H * N * d, H * N * N
