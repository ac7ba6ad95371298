// Internal declarations shared by the library's translation units (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>
#include "../../include/cascade.h"

// One tile of packed rows that never straddles a shard boundary.  sub_min/sub_max hold
// the smallest / largest token position of each 16-row granule of the tile (granules
// beyond n_rows hold min = INT_MAX, max = INT_MIN).
struct CascadeTile {
    int32_t row_start;   // first packed row
    int32_t n_rows;      // rows in this tile (<= granule)
    int32_t shard;       // shard id
    int32_t pmin;        // min position over the tile
    int32_t pmax;        // max position over the tile
    int32_t index;       // index of the tile in packed order (kept when the list is reordered)
    int32_t pad[2];
    int32_t sub_min[16];
    int32_t sub_max[16];
};

struct CascadeTileList {
    int32_t granule = 0;
    int32_t count = 0;
    CascadeTile *dev = nullptr;           // packed order
    CascadeTile *dev_by_pmin = nullptr;   // the same tiles ordered by smallest position (stable)
    CascadeTile *dev_by_shard_pmin = nullptr;   // packed order of shards, each shard's tiles by smallest position
    CascadeTile *dev_by_pmax_desc = nullptr;    // the same tiles ordered by largest position, descending (stable)
    int32_t *shard_first = nullptr;   // device: [n_shards + 1] first tile index of each shard
    int32_t *shard_first_host = nullptr;
    // positions of the tile's rows, granule values per tile (tile `index` at index * granule), rows past the
    // tile's end hold 2^30; built for the 64-row list only (the key/value tiles of the attention kernels)
    int32_t *pos_padded = nullptr;
};

struct cascade_plan {
    int32_t batch, seq_len, n_shards, mask_kind;
    int device;
    // host copies
    int32_t *perm_h, *inv_perm_h, *offsets_h, *pos_packed_h;
    // device copies
    int32_t *perm_d, *inv_perm_d, *offsets_d, *pos_packed_d;
    int32_t max_abs_pos;        // largest |position|
    int32_t last_token;         // token with the largest position (lowest index among equals)
    int32_t *last_rows_d;       // [2][batch]: row of that token in every sequence, packed order then original order
    CascadeTileList tiles[4];   // granules 32, 64, 128, 256
    // Key/value partition S when it differs from the row partition R (Section 5.1; the m-split of
    // Section 6.4): a plan of its own over the same tokens, plus the map from its packed rows to
    // this plan's packed rows.  nullptr: S = R.
    cascade_plan *kv;
    int32_t *kv_to_row_h, *kv_to_row_d;
    // Causal plans: the same tokens as one shard in ascending position (ties by token index), with its tile
    // lists, and the map from its rows to this plan's packed rows.  The fused attention kernel may walk queries
    // and keys in that order (the merge over key/value shards does not depend on how the keys are grouped):
    // a tile then covers neighbouring positions and only the tiles on the diagonal hold masked scores.
    cascade_plan *sorted;
    int32_t *sorted_to_row_d;
};

// the partition that shards keys and values (the plan itself when S = R)
static inline const cascade_plan *kv_plan(const cascade_plan *p) { return p->kv ? p->kv : p; }

static inline const CascadeTileList &plan_tiles(const cascade_plan *p, int granule) {
    return p->tiles[granule == 32 ? 0 : granule == 64 ? 1 : granule == 128 ? 2 : 3];
}

void cascade_set_hip_error(hipError_t e);

#define CASCADE_HIP_TRY(expr)                                   \
    do {                                                        \
        hipError_t _e = (expr);                                 \
        if (_e != hipSuccess) { cascade_set_hip_error(_e); return CASCADE_EHIP; } \
    } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic LDS limit once per device (the attribute is per device; setting it again
// is harmless, so concurrent first calls need no lock).  `done` is a bit mask of devices, one per kernel.
static inline hipError_t ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev < 64 ? (1ull << dev) : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// ---------------------------------------------------------------------------- internal launchers
// Row map convention: map == nullptr -> identity; else global row = b * seq_len + map[r % seq_len].
struct RowMap {
    const int32_t *map;
    int32_t seq_len;
};

struct GemmArgs {
    int32_t dtype;
    int32_t M, N, K;                 // N: output columns (SWIGLU: of the product)
    const void *X;
    const void *W[3];                // weight segments stacked along the output axis
    int32_t seg_end[3];              // exclusive end column of each segment (unused segments: N)
    const void *bias[3];             // per segment, may be null
    const void *W_up;                // SWIGLU second operand
    const void *residual;
    void *Y;
    int64_t ldx, ldy, ldres;         // row strides in elements
    RowMap xmap, ymap, rmap;
    int32_t epilogue;
    // Rotary embedding applied to the output in the epilogue (bf16, see gemm_bf16_rope_fusable): cos | sin of the
    // angles of every row, [M][rope_head_dim] fp32, rows in the order of the GEMM's rows; columns below rope_cols
    // are rotated (half-split pairs inside heads of rope_head_dim columns).  nullptr: no rotation.
    const float *rope_table;
    int32_t rope_cols, rope_head_dim;
    // Scratch for a reduction split over two workgroups per tile (bf16, see gemm_bf16_splitk_bytes): fp32 partial
    // tiles, and the per-tile ticket and flag words, GEMM_SPLITK_SYNC_WORDS of them, which must have been zero when
    // the first launch that uses them started (launches that share them run one after the other).  nullptr: the
    // launch does not split.
    float *sk_partial;
    size_t sk_partial_bytes;
    uint32_t *sk_sync;
};
constexpr int GEMM_SPLITK_MAX_TILES = 256;
constexpr int GEMM_SPLITK_SYNC_WORDS = 2 * GEMM_SPLITK_MAX_TILES;

int32_t launch_gemm_bf16(const GemmArgs &a, hipStream_t s);
bool gemm_bf16_rope_fusable(const GemmArgs &a);
// Bytes of GemmArgs::sk_partial that a launch of this shape would use for a split reduction; 0 when it would not
// split (the shape fills the CUs without, or the split kernel does not take it).
size_t gemm_bf16_splitk_bytes(int32_t M, int32_t N, int32_t K);
int32_t launch_gemm_f32(const GemmArgs &a, hipStream_t s);

struct NormArgs {
    int32_t dtype, rows, D, kind;
    float eps;
    const void *x; const void *gain; const void *bias; void *y;
    RowMap xmap;                     // gather on the read
    RowMap ymap;                     // scatter on the write
    // Optional by-product: cos | sin of the rotary angles of row r (position rope_pos[r % rope_seq_len]),
    // [rows][rope_head_dim] fp32, written by the workgroup that normalises row r.  nullptr: none.
    float *rope_table;
    const int32_t *rope_pos;
    int32_t rope_seq_len, rope_head_dim;
    float rope_theta;
    // Optional: n_zero_words words cleared by the launch (flags of the split-reduction GEMMs later in the stream)
    uint32_t *zero_words;
    int32_t n_zero_words;
};
int32_t launch_norm(const NormArgs &a, hipStream_t s);
// k, v rows of a packed [T, ld] activation (columns k_col0 .. and v_col0 .., H_kv heads of d) -> cache slabs
// [B, H_kv, n_shards, cap, d]; shard k holds rows offsets[k] .. offsets[k+1] of the (kv) packed order, row_of
// maps those to rows of the activation (nullptr: identity); shard_len [B, n_shards] receives the sizes
struct KvCacheArgs {
    int32_t dtype, B, N, Hkv, d, n_shards, cap;
    const void *act; int64_t ld; int32_t k_col0, v_col0;
    const int32_t *offsets, *row_of;
    void *k_cache, *v_cache; int32_t *shard_len;
};
int32_t launch_kv_to_cache(const KvCacheArgs &a, hipStream_t s);
// token_out[r] = lowest index of the largest element of row r of x [rows, ld] (first `vocab` columns)
int32_t launch_argmax_rows(int32_t dtype, const void *x, int64_t ld, int32_t rows, int32_t vocab, int32_t *token_out,
                           hipStream_t s);

struct RopeArgs {
    int32_t dtype, rows, seq_len;    // rows = B * N packed rows
    int32_t n_rope_heads, head_dim;  // heads [0, n_rope_heads) of each row are rotated
    int64_t ld;                      // row stride (elements)
    float theta;
    const int32_t *pos_packed;       // [seq_len]
    void *x;                         // in place
    int32_t max_pos;                 // largest |position| of the plan (the fast bf16 path needs < 2^24)
};
int32_t launch_rope(const RopeArgs &a, hipStream_t s);

struct AttnArgs {
    int32_t dtype, B, H, Hkv, d;
    float scale;
    int32_t mask_kind;
    const void *q, *k, *v;
    int64_t qs_b, qs_h, qs_n, ks_b, ks_h, ks_n;     // element strides; k and v share theirs
    const int32_t *q_rowmap, *kv_rowmap;   // packed row -> row in q / k,v (nullptr: identity)
    int32_t fused;                   // 1: running merge over all shards, write o; 0: per-shard partials
    int32_t u_mode;
    float *m, *e, *u;                // partials (fused == 0)
    void *o; int64_t o_ld;           // fused output [B, N, H*d], row map below
    const int32_t *o_rowmap;
    void *workspace; size_t workspace_bytes;
};
size_t attn_bf16_workspace_bytes(const cascade_plan *p, int32_t B, int32_t Hkv, int32_t d);
int32_t launch_attn_bf16(const cascade_plan *p, const AttnArgs &a, hipStream_t s);
int32_t launch_attn_f32(const cascade_plan *p, const AttnArgs &a, hipStream_t s);

struct MergeArgs {
    int32_t dtype, B, H, d, n_shards, N, u_mode;
    const float *m, *e, *u;
    void *o; int64_t o_ld;
    const int32_t *o_rowmap;         // packed row -> output row (nullptr: identity)
    float *lse;
};
int32_t launch_merge(const MergeArgs &a, hipStream_t s);
