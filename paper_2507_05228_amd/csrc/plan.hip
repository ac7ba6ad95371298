// Shard plan: the partition of [N] (Section 5.1) as index maps and tile lists.
// Host integer work only; the results are copied to the device once.
#include <algorithm>
#include <climits>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>
#include "common.h"

static thread_local int32_t g_last_hip_error = 0;

void cascade_set_hip_error(hipError_t e) { g_last_hip_error = (int32_t)e; }

extern "C" int32_t cascade_last_hip_error(void) { return g_last_hip_error; }

static void free_plan(cascade_plan *p) {
    if (!p) return;
    free_plan(p->kv);
    free_plan(p->sorted);
    if (p->sorted_to_row_d) (void)hipFree(p->sorted_to_row_d);
    free(p->kv_to_row_h);
    if (p->kv_to_row_d) (void)hipFree(p->kv_to_row_d);
    free(p->perm_h); free(p->inv_perm_h); free(p->offsets_h); free(p->pos_packed_h);
    if (p->perm_d) (void)hipFree(p->perm_d);
    if (p->inv_perm_d) (void)hipFree(p->inv_perm_d);
    if (p->offsets_d) (void)hipFree(p->offsets_d);
    if (p->pos_packed_d) (void)hipFree(p->pos_packed_d);
    if (p->last_rows_d) (void)hipFree(p->last_rows_d);
    for (auto &t : p->tiles) {
        if (t.dev) (void)hipFree(t.dev);
        if (t.dev_by_pmin) (void)hipFree(t.dev_by_pmin);
        if (t.dev_by_shard_pmin) (void)hipFree(t.dev_by_shard_pmin);
        if (t.dev_by_pmax_desc) (void)hipFree(t.dev_by_pmax_desc);
        if (t.shard_first) (void)hipFree(t.shard_first);
        if (t.pos_padded) (void)hipFree(t.pos_padded);
        free(t.shard_first_host);
    }
    delete p;
}

template <typename T>
static hipError_t to_device(T **dst, const T *src, size_t n) {
    *dst = nullptr;
    size_t bytes = (n ? n : 1) * sizeof(T);
    hipError_t e = hipMalloc((void **)dst, bytes);
    if (e != hipSuccess) return e;
    if (n) e = hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice);
    return e;
}

// Tiles of at most `granule` packed rows, each inside one shard, in packed order.
static hipError_t build_tiles(cascade_plan *p, CascadeTileList &out, int granule) {
    std::vector<CascadeTile> tiles;
    std::vector<int32_t> first(p->n_shards + 1, 0);
    for (int j = 0; j < p->n_shards; ++j) {
        first[j] = (int32_t)tiles.size();
        for (int r = p->offsets_h[j]; r < p->offsets_h[j + 1]; r += granule) {
            CascadeTile t;
            memset(&t, 0, sizeof(t));
            t.row_start = r;
            t.n_rows = std::min(granule, p->offsets_h[j + 1] - r);
            t.shard = j;
            t.index = (int32_t)tiles.size();
            t.pmin = INT_MAX;
            t.pmax = INT_MIN;
            for (int g = 0; g < 16; ++g) { t.sub_min[g] = INT_MAX; t.sub_max[g] = INT_MIN; }
            for (int i = 0; i < t.n_rows; ++i) {
                int pos = p->pos_packed_h[r + i];
                int g = i / 16;
                t.sub_min[g] = std::min(t.sub_min[g], pos);
                t.sub_max[g] = std::max(t.sub_max[g], pos);
                t.pmin = std::min(t.pmin, pos);
                t.pmax = std::max(t.pmax, pos);
            }
            tiles.push_back(t);
        }
    }
    first[p->n_shards] = (int32_t)tiles.size();
    out.granule = granule;
    out.count = (int32_t)tiles.size();
    out.shard_first_host = (int32_t *)malloc(first.size() * sizeof(int32_t));
    if (!out.shard_first_host) return hipErrorOutOfMemory;
    memcpy(out.shard_first_host, first.data(), first.size() * sizeof(int32_t));
    hipError_t e = to_device(&out.dev, tiles.data(), tiles.size());
    if (e != hipSuccess) return e;
    std::vector<CascadeTile> sorted(tiles);
    std::stable_sort(sorted.begin(), sorted.end(), [](const CascadeTile &x, const CascadeTile &y) { return x.pmin < y.pmin; });
    e = to_device(&out.dev_by_pmin, sorted.data(), sorted.size());
    if (e != hipSuccess) return e;
    sorted = tiles;                                       // shard ranges kept, each ordered by smallest position
    for (int j = 0; j < p->n_shards; ++j)
        std::stable_sort(sorted.begin() + first[j], sorted.begin() + first[j + 1],
                         [](const CascadeTile &x, const CascadeTile &y) { return x.pmin < y.pmin; });
    e = to_device(&out.dev_by_shard_pmin, sorted.data(), sorted.size());
    if (e != hipSuccess) return e;
    sorted = tiles;
    std::stable_sort(sorted.begin(), sorted.end(), [](const CascadeTile &x, const CascadeTile &y) { return x.pmax > y.pmax; });
    e = to_device(&out.dev_by_pmax_desc, sorted.data(), sorted.size());
    if (e != hipSuccess) return e;
    if (granule == 64) {
        // (2^30: above every position the fused kernel accepts, and "limit - 2^30" cannot overflow for any limit it uses)
        std::vector<int32_t> padded(tiles.size() * 64, 1 << 30);
        for (size_t t = 0; t < tiles.size(); ++t)
            for (int i = 0; i < tiles[t].n_rows; ++i) padded[t * 64 + i] = p->pos_packed_h[tiles[t].row_start + i];
        e = to_device(&out.pos_padded, padded.data(), padded.size());
        if (e != hipSuccess) return e;
    }
    return to_device(&out.shard_first, first.data(), first.size());
}

static int32_t complete_plan(cascade_plan *p, const int32_t *positions_host);
static int32_t build_sorted_view(cascade_plan *p, const int32_t *positions_host);

static int32_t build_plan(cascade_plan **out, int32_t batch, int32_t seq_len, int32_t n_shards,
                          const int32_t *token_to_shard_host, const int32_t *positions_host, int32_t mask_kind,
                          bool with_sorted_view) {
    if (!out) return CASCADE_EINVAL;
    *out = nullptr;
    if (!token_to_shard_host || batch <= 0 || seq_len <= 0 || n_shards <= 0) return CASCADE_EINVAL;
    if (mask_kind != CASCADE_MASK_NONE && mask_kind != CASCADE_MASK_CAUSAL) return CASCADE_EINVAL;
    if ((int64_t)batch * seq_len > INT32_MAX / 2) return CASCADE_EUNSUPPORTED;
    for (int t = 0; t < seq_len; ++t)
        if (token_to_shard_host[t] < 0 || token_to_shard_host[t] >= n_shards) return CASCADE_EASSIGN;

    cascade_plan *p = new (std::nothrow) cascade_plan();
    if (!p) return CASCADE_EINVAL;
    memset(p, 0, sizeof(*p));
    p->batch = batch; p->seq_len = seq_len; p->n_shards = n_shards; p->mask_kind = mask_kind;
    p->perm_h = (int32_t *)malloc(sizeof(int32_t) * seq_len);
    p->inv_perm_h = (int32_t *)malloc(sizeof(int32_t) * seq_len);
    p->offsets_h = (int32_t *)malloc(sizeof(int32_t) * (n_shards + 1));
    p->pos_packed_h = (int32_t *)malloc(sizeof(int32_t) * seq_len);
    if (!p->perm_h || !p->inv_perm_h || !p->offsets_h || !p->pos_packed_h) { free_plan(p); return CASCADE_EINVAL; }

    // Counting sort by shard id: stable, so rows inside a shard stay in ascending token index.
    memset(p->offsets_h, 0, sizeof(int32_t) * (n_shards + 1));
    for (int t = 0; t < seq_len; ++t) p->offsets_h[token_to_shard_host[t] + 1]++;
    for (int j = 0; j < n_shards; ++j) p->offsets_h[j + 1] += p->offsets_h[j];
    {
        std::vector<int32_t> cursor(p->offsets_h, p->offsets_h + n_shards);
        for (int t = 0; t < seq_len; ++t) {
            int r = cursor[token_to_shard_host[t]]++;
            p->perm_h[r] = t;
            p->inv_perm_h[t] = r;
        }
    }
    const int32_t st = complete_plan(p, positions_host);
    if (st != CASCADE_OK) { free_plan(p); return st; }
    if (with_sorted_view && mask_kind == CASCADE_MASK_CAUSAL) {
        const int32_t st2 = build_sorted_view(p, positions_host);
        if (st2 != CASCADE_OK) { free_plan(p); return st2; }
    }
    *out = p;
    return CASCADE_OK;
}

// Positions of the packed rows, the last token, device copies and tile lists of a plan whose perm_h, inv_perm_h and
// offsets_h are filled in.
static int32_t complete_plan(cascade_plan *p, const int32_t *positions_host) {
    const int32_t batch = p->batch, seq_len = p->seq_len, n_shards = p->n_shards;
    for (int r = 0; r < seq_len; ++r) {
        p->pos_packed_h[r] = positions_host ? positions_host[p->perm_h[r]] : p->perm_h[r];
        const int64_t ap = std::llabs((int64_t)p->pos_packed_h[r]);
        p->max_abs_pos = (int32_t)std::min<int64_t>(std::max<int64_t>(p->max_abs_pos, ap), INT32_MAX);
    }

    for (int t = 1; t < seq_len; ++t) {
        const int32_t pt = positions_host ? positions_host[t] : t;
        const int32_t pl = positions_host ? positions_host[p->last_token] : p->last_token;
        if (pt > pl) p->last_token = t;
    }
    std::vector<int32_t> last_rows(2 * (size_t)batch);
    for (int b = 0; b < batch; ++b) {
        last_rows[b] = b * seq_len + p->inv_perm_h[p->last_token];
        last_rows[batch + b] = b * seq_len + p->last_token;
    }

    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess) e = to_device(&p->last_rows_d, last_rows.data(), 2 * batch);
    if (e == hipSuccess) e = to_device(&p->perm_d, p->perm_h, seq_len);
    if (e == hipSuccess) e = to_device(&p->inv_perm_d, p->inv_perm_h, seq_len);
    if (e == hipSuccess) e = to_device(&p->offsets_d, p->offsets_h, n_shards + 1);
    if (e == hipSuccess) e = to_device(&p->pos_packed_d, p->pos_packed_h, seq_len);
    static const int granules[4] = {32, 64, 128, 256};
    for (int g = 0; g < 4 && e == hipSuccess; ++g) e = build_tiles(p, p->tiles[g], granules[g]);
    if (e != hipSuccess) { cascade_set_hip_error(e); return CASCADE_EHIP; }
    return CASCADE_OK;
}

// The position-sorted one-shard view of a causal plan (see cascade_plan::sorted).
static int32_t build_sorted_view(cascade_plan *p, const int32_t *positions_host) {
    const int32_t N = p->seq_len;
    cascade_plan *v = new (std::nothrow) cascade_plan();
    if (!v) return CASCADE_EINVAL;
    memset(v, 0, sizeof(*v));
    p->sorted = v;                                           // freed with p from here on
    v->batch = p->batch; v->seq_len = N; v->n_shards = 1; v->mask_kind = p->mask_kind;
    v->perm_h = (int32_t *)malloc(sizeof(int32_t) * N);
    v->inv_perm_h = (int32_t *)malloc(sizeof(int32_t) * N);
    v->offsets_h = (int32_t *)malloc(sizeof(int32_t) * 2);
    v->pos_packed_h = (int32_t *)malloc(sizeof(int32_t) * N);
    if (!v->perm_h || !v->inv_perm_h || !v->offsets_h || !v->pos_packed_h) return CASCADE_EINVAL;
    for (int t = 0; t < N; ++t) v->perm_h[t] = t;
    if (positions_host)
        std::stable_sort(v->perm_h, v->perm_h + N, [&](int32_t x, int32_t y) { return positions_host[x] < positions_host[y]; });
    for (int r = 0; r < N; ++r) v->inv_perm_h[v->perm_h[r]] = r;
    v->offsets_h[0] = 0; v->offsets_h[1] = N;
    const int32_t st = complete_plan(v, positions_host);
    if (st != CASCADE_OK) return st;
    std::vector<int32_t> to_row(N);
    for (int r = 0; r < N; ++r) to_row[r] = p->inv_perm_h[v->perm_h[r]];
    const hipError_t e = to_device(&p->sorted_to_row_d, to_row.data(), N);
    if (e != hipSuccess) { cascade_set_hip_error(e); return CASCADE_EHIP; }
    return CASCADE_OK;
}

extern "C" int32_t cascade_plan_create(cascade_plan **out, int32_t batch, int32_t seq_len, int32_t n_shards,
                                       const int32_t *token_to_shard_host, const int32_t *positions_host,
                                       int32_t mask_kind) {
    return build_plan(out, batch, seq_len, n_shards, token_to_shard_host, positions_host, mask_kind, true);
}

extern "C" int32_t cascade_plan_create_rs(cascade_plan **out, int32_t batch, int32_t seq_len, int32_t n_row_shards,
                                          const int32_t *token_to_row_shard_host, int32_t n_kv_shards,
                                          const int32_t *token_to_kv_shard_host, const int32_t *positions_host,
                                          int32_t mask_kind) {
    if (!out) return CASCADE_EINVAL;
    *out = nullptr;
    if (!token_to_kv_shard_host || n_kv_shards <= 0) return CASCADE_EINVAL;
    cascade_plan *p = nullptr;
    int32_t st = build_plan(&p, batch, seq_len, n_row_shards, token_to_row_shard_host, positions_host, mask_kind, true);
    if (st != CASCADE_OK) return st;
    st = build_plan(&p->kv, batch, seq_len, n_kv_shards, token_to_kv_shard_host, positions_host, mask_kind, false);
    if (st != CASCADE_OK) { free_plan(p); return st; }
    p->kv_to_row_h = (int32_t *)malloc(sizeof(int32_t) * seq_len);
    if (!p->kv_to_row_h) { free_plan(p); return CASCADE_EINVAL; }
    for (int r = 0; r < seq_len; ++r) p->kv_to_row_h[r] = p->inv_perm_h[p->kv->perm_h[r]];
    hipError_t e = to_device(&p->kv_to_row_d, p->kv_to_row_h, seq_len);
    if (e != hipSuccess) { cascade_set_hip_error(e); free_plan(p); return CASCADE_EHIP; }
    *out = p;
    return CASCADE_OK;
}

extern "C" int32_t cascade_plan_kv_maps_host(const cascade_plan *plan, int32_t *n_kv_shards, const int32_t **kv_perm_host,
                                             const int32_t **kv_offsets_host, const int32_t **kv_to_row_host) {
    if (!plan) return CASCADE_EINVAL;
    const cascade_plan *k = kv_plan(plan);
    if (n_kv_shards) *n_kv_shards = k->n_shards;
    if (kv_perm_host) *kv_perm_host = k->perm_h;
    if (kv_offsets_host) *kv_offsets_host = k->offsets_h;
    if (kv_to_row_host) *kv_to_row_host = plan->kv ? plan->kv_to_row_h : nullptr;
    return CASCADE_OK;
}

// ---------------------------------------------------------------------------- (c, delta) plans
// Section 6 ((c, delta)-sequences): shard i of a (c, delta)-sharding holds the tokens {i c .. i c + c - 1} + multiples
// of delta (0-based), i.e. token t goes to shard (t mod delta) div c; ceil(delta / c) shards.
extern "C" int32_t cascade_cdelta_assignment(int32_t seq_len, int32_t c, int32_t delta, int32_t *token_to_shard_host,
                                             int32_t *n_shards) {
    if (!token_to_shard_host || seq_len <= 0 || c <= 0 || delta <= 0) return CASCADE_EINVAL;
    for (int t = 0; t < seq_len; ++t) token_to_shard_host[t] = (t % delta) / c;
    if (n_shards) *n_shards = (delta + c - 1) / c;
    return CASCADE_OK;
}

// Section 6.4 (AttnNode Full Security, m-split; its N = 18 example fixes the reading): every row
// shard R_i, sorted, is dealt round-robin into m pieces; piece x of
// shard i (0-based) becomes kv shard m i + x, so beta = m alpha and pairwise coverage is kept.
extern "C" int32_t cascade_m_split(int32_t seq_len, int32_t n_row_shards, const int32_t *token_to_row_shard_host,
                                   int32_t m, int32_t *token_to_kv_shard_host) {
    if (!token_to_row_shard_host || !token_to_kv_shard_host || seq_len <= 0 || n_row_shards <= 0 || m <= 0)
        return CASCADE_EINVAL;
    if ((int64_t)n_row_shards * m > INT32_MAX) return CASCADE_EUNSUPPORTED;
    std::vector<int32_t> seen(n_row_shards, 0);          // rank of the token inside its sorted row shard
    for (int t = 0; t < seq_len; ++t) {
        const int32_t i = token_to_row_shard_host[t];
        if (i < 0 || i >= n_row_shards) return CASCADE_EASSIGN;
        token_to_kv_shard_host[t] = m * i + seen[i]++ % m;
    }
    return CASCADE_OK;
}

// ---------------------------------------------------------------------------- cost model
// Equation 1 (Communication Analysis appendix): bytes per layer moved between CompNodes and
// AttnNodes.  Stage A ships every q row to beta AttnNodes and every k, v row to beta AttnNodes;
// stage B ships m, e (1 + 1 values) and u (d values) per head and row back from beta AttnNodes.
// Rounds per layer: at most 2 alpha beta^2 in general, 2 beta^2 for (c, delta)-sharding with an m-split.
extern "C" int32_t cascade_comm_cost(int32_t n_row_shards, int32_t n_kv_shards, int32_t m_split_scheme,
                                     int32_t bytes_per_value, int32_t head_dim, int32_t n_heads, int32_t n_kv_heads,
                                     int64_t seq_len, int64_t *stage_a_bytes, int64_t *stage_b_bytes,
                                     int64_t *rounds) {
    if (n_row_shards <= 0 || n_kv_shards <= 0 || bytes_per_value <= 0 || head_dim <= 0 || n_heads <= 0 ||
        n_kv_heads <= 0 || seq_len <= 0)
        return CASCADE_EINVAL;
    const int64_t beta = n_kv_shards, F = bytes_per_value, d = head_dim;
    if (stage_a_bytes) *stage_a_bytes = beta * F * d * (n_heads + 2 * (int64_t)n_kv_heads) * seq_len;
    if (stage_b_bytes) *stage_b_bytes = beta * F * (d + 2) * n_heads * seq_len;
    if (rounds) *rounds = m_split_scheme ? 2 * beta * beta : 2 * (int64_t)n_row_shards * beta * beta;
    return CASCADE_OK;
}

// Equation 2 (Theoretical Costs; derived in the Communication Analysis appendix): with perfect parallel
// transport a stage lasts one latency plus the transfer of the node that sends most.  Stage A: the
// CompNode with the largest row shard ships each row's q, k, v to beta AttnNodes; stage B: an AttnNode
// of the largest key/value shard ships u, m, e of its rows back.
extern "C" int32_t cascade_comm_time(const cascade_plan *plan, int32_t n_kv_shards, int32_t max_row_shard,
                                     int32_t max_kv_shard, int32_t bytes_per_value, int32_t head_dim,
                                     int32_t n_heads, int32_t n_kv_heads, double latency_s,
                                     double bandwidth_bytes_per_s, double *stage_a_s, double *stage_b_s,
                                     double *total_s) {
    if (plan) {                                    // shard sizes from the plan's two partitions
        const cascade_plan *kvp = kv_plan(plan);
        n_kv_shards = kvp->n_shards;
        max_row_shard = max_kv_shard = 0;
        for (int i = 0; i < plan->n_shards; ++i)
            max_row_shard = std::max(max_row_shard, plan->offsets_h[i + 1] - plan->offsets_h[i]);
        for (int j = 0; j < kvp->n_shards; ++j)
            max_kv_shard = std::max(max_kv_shard, kvp->offsets_h[j + 1] - kvp->offsets_h[j]);
    }
    if (n_kv_shards <= 0 || max_row_shard < 0 || max_kv_shard < 0 || bytes_per_value <= 0 || head_dim <= 0 ||
        n_heads <= 0 || n_kv_heads <= 0 || !(latency_s >= 0.0) || !(bandwidth_bytes_per_s > 0.0))
        return CASCADE_EINVAL;
    const double beta = n_kv_shards, F = bytes_per_value, d = head_dim;
    const double a = latency_s + beta * F * d * (n_heads + 2.0 * n_kv_heads) / bandwidth_bytes_per_s * max_row_shard;
    const double b = latency_s + F * (d + 2.0) * n_heads / bandwidth_bytes_per_s * max_kv_shard;
    if (stage_a_s) *stage_a_s = a;
    if (stage_b_s) *stage_b_s = b;
    if (total_s) *total_s = a + b;
    return CASCADE_OK;
}

extern "C" int32_t cascade_plan_maps(const cascade_plan *plan, const int32_t **perm_dev,
                                     const int32_t **inv_perm_dev, const int32_t **offsets_dev) {
    if (!plan) return CASCADE_EINVAL;
    if (perm_dev) *perm_dev = plan->perm_d;
    if (inv_perm_dev) *inv_perm_dev = plan->inv_perm_d;
    if (offsets_dev) *offsets_dev = plan->offsets_d;
    return CASCADE_OK;
}

extern "C" int32_t cascade_plan_maps_host(const cascade_plan *plan, const int32_t **perm_host,
                                          const int32_t **inv_perm_host, const int32_t **offsets_host) {
    if (!plan) return CASCADE_EINVAL;
    if (perm_host) *perm_host = plan->perm_h;
    if (inv_perm_host) *inv_perm_host = plan->inv_perm_h;
    if (offsets_host) *offsets_host = plan->offsets_h;
    return CASCADE_OK;
}

extern "C" void cascade_plan_destroy(cascade_plan *plan) { free_plan(plan); }
