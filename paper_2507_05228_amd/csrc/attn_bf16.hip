// bf16 partial attention on the gfx950 matrix cores (Algorithm 3) and its fused variant, which
// keeps Algorithm 4's running maximum n, weight sum w and output o in registers while it walks the
// key/value shards (same arithmetic as the post-pass, with the maximum updated online).
//
// Work split: a workgroup of 8 wavefronts (2 per SIMD, so one wavefront's softmax arithmetic
// overlaps the other's MFMAs) owns one tile of packed query rows (never straddling a shard) for up
// to 4 query heads that share one key/value head: the K / V tiles staged in LDS are reused by all
// of them (GQA).  A wavefront owns 32 query rows (two 16-row blocks) of one head.
//
// MFMA arrangement (16x16x32 bf16): the score block is computed TRANSPOSED, S^T = K Q^T, so a lane
// holds ONE query row (column lane%16) and 4 keys of it per 16x16 block.  Row maximum and sum of
// exponentials are register-local plus exchanges with lanes ^16 and ^32, and rescaling the output
// accumulator is a per-lane multiply.  The second product is O^T = V^T P^T: the exponentials go
// from the accumulator layout straight into the B operand (the contraction index is permuted the
// same way on both operands), and V^T comes from a transposed copy of V built once per call, so
// both LDS tiles are read with vector loads.
//
// Tiles of 64 keys go from L2/HBM straight into LDS (buffer loads that write LDS, zero for rows
// past a ragged tile), two stages; rows are stored without padding, 16-byte chunk c of row r at
// slot c ^ swizzle(r), so operand reads are bank-conflict free.
//
// Masking: key visible iff position[key] <= position[query] (original token positions).  Tiles and
// 16x16 blocks whose smallest key position exceeds the largest query position are skipped; blocks
// that are fully visible skip the compare.
#include <climits>
#include <cstdlib>
#include <type_traits>
#include "attn_bf16.h"

// ---------------------------------------------------------------------------- V -> V^T (tile order)
// vt[b][g][c][64 t + col(i)] = v[b][g][row(tile t, i)][c] for i < n_rows(t), zero for the padding of a
// ragged tile.  Column 64 t of V^T is therefore 16-byte aligned for every key/value tile t.  Inside
// a tile the keys are permuted so that the 8 keys one lane feeds to an MFMA k-step of O^T += V^T P^T
// are contiguous: key i = 32 s + 16 jh + 4 g + jl sits at col(i) = 32 s + 8 g + 4 jh + jl (the P^T
// operand of lane group g is built from accumulator registers jl of score blocks 2s + jh).
template <int D>
__global__ __launch_bounds__(256) void vtranspose_kernel(const bf16_t *__restrict__ v, bf16_t *__restrict__ vt,
                                                         int64_t vs_b, int64_t vs_h, int64_t vs_n, int npad,
                                                         int Hkv, const CascadeTile *__restrict__ kvtiles,
                                                         const int32_t *__restrict__ rowmap,
                                                         const bf16_t *__restrict__ k, bf16_t *__restrict__ kp, int N) {
    __shared__ bf16_t tile[64][D + 2];
    const int t = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int r0 = kvtiles[t].row_start, nr = kvtiles[t].n_rows;
    const bf16_t *vb = v + b * vs_b + g * vs_h;
    constexpr int CPR = D / 8;
    // The tile's rows: every thread takes the same (row, 16-byte chunk) pairs of K and of V.  All row-map lookups go
    // out first, then all loads: two memory round trips per workgroup instead of two per pair (a 16 MB pass that took
    // 8 us with the lookups and loads of a pair chasing each other).
    constexpr int IT = 64 * CPR / 256;
    static_assert(64 * CPR % 256 == 0, "whole passes");
    int rr_[IT], ch_[IT];
    int64_t src[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        const int id = threadIdx.x + 256 * i;
        rr_[i] = id / CPR; ch_[i] = id % CPR;
        const int r = r0 + (rr_[i] < nr ? rr_[i] : 0);
        src[i] = rowmap ? rowmap[r] : r;
    }
    // On the side (kp given; k has v's strides): the tile's K rows into packed order, kp[b][g][r][D], for callers
    // whose K is in another row order, so that the attention kernel's tile loads never chase a row map.
    bf16x8 kval[IT], vval[IT];
    if (kp) {
        const bf16_t *kb = k + b * vs_b + g * vs_h;
#pragma unroll
        for (int i = 0; i < IT; ++i) kval[i] = *(const bf16x8 *)(kb + src[i] * vs_n + ch_[i] * 8);
    }
#pragma unroll
    for (int i = 0; i < IT; ++i) vval[i] = *(const bf16x8 *)(vb + src[i] * vs_n + ch_[i] * 8);
    if (kp) {
#pragma unroll
        for (int i = 0; i < IT; ++i)
            if (rr_[i] < nr) *(bf16x8 *)(kp + (((int64_t)b * Hkv + g) * N + r0 + rr_[i]) * D + ch_[i] * 8) = kval[i];
    }
#pragma unroll
    for (int i = 0; i < IT; ++i) {
#pragma unroll
        for (int x = 0; x < 8; ++x) tile[rr_[i]][ch_[i] * 8 + x] = rr_[i] < nr ? vval[i][x] : (bf16_t)0.f;
    }
    __syncthreads();
    bf16_t *ob = vt + ((int64_t)b * Hkv + g) * D * npad + (int64_t)t * 64;
    for (int id = threadIdx.x; id < D * 8; id += 256) {
        int c = id / 8, ch = id % 8;
        bf16x8 val;
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] = tile[32 * (ch >> 2) + 16 * (i >> 2) + 4 * (ch & 3) + (i & 3)][c];
        *(bf16x8 *)(ob + (int64_t)c * npad + ch * 8) = val;
    }
}

// ---------------------------------------------------------------------------- attention
// NWV = 8: the workgroup described above.  NWV = 4: half of it (one wavefront per SIMD, up to 128 query rows
// of one head), for plans whose shards are too short to give 8 wavefronts rows; two such workgroups share a
// CU when their LDS fits (head dimension 64) and overlap each other's phases instead.
template <int D, int NWV>
__global__ __launch_bounds__(NWV * 64) void attn_bf16_kernel(AttnBf16Params p) {
    constexpr int TQ = 2;                              // 16-row query blocks per wavefront
    constexpr int KS = D / 32;                         // k-steps of the score product
    constexpr int DB = D / 16;                         // 16-row blocks of O^T
    constexpr int K_ROW = D * 2;                       // bytes per K row in LDS (256 or 128)
    constexpr int K_RPI = 1024 / K_ROW;                // K rows filled by one direct-to-LDS instruction
    constexpr int K_CPR = K_ROW / 16;                  // 16-byte chunks per K row
    constexpr int K_BYTES = KV_TILE * K_ROW, V_BYTES = D * 128;
    constexpr int STAGE = K_BYTES + V_BYTES + KV_TILE * 4;   // K tile, V^T tile, key positions
    constexpr int K_INSTR = KV_TILE / K_RPI / NWV;     // per wavefront; 8 wavefronts: 2 (D=128) or 1 (D=64)
    constexpr int V_INSTR = D / 8 / NWV;               // 2 or 1
    static_assert(NWV == 4 || NWV == 8, "one or two wavefronts per SIMD");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g4 = lane >> 4;
    const int hpb = p.hpb;
    const int hsel = wave % hpb, rg = wave / hpb;
    const int rep = p.H / p.Hkv;
    const int hblocks = rep / hpb;
    // Workgroups of one query tile are neighbours in launch order (the kv heads fastest: with 8 of them each
    // XCD serves one head's K and V), and the tiles come heaviest first.
    const int q_tile = blockIdx.x / p.gy, by = blockIdx.x % p.gy;
    const int b = by / (p.Hkv * hblocks);
    const int gh = by % (p.Hkv * hblocks);
    const int g = gh / hblocks;
    const int h = g * rep + (gh % hblocks) * hpb + hsel;
    const int kk = p.fused ? 0 : blockIdx.z;

    const tile_cptr kvtiles = (tile_cptr)p.kvtiles;
    const tile_cptr qtp = (tile_cptr)p.qtiles + q_tile;
    const int q_row_start = qtp->row_start, q_n_rows = qtp->n_rows, q_pmax = qtp->pmax;
    const int wrow0 = rg * 16 * TQ;                    // first row of this wavefront inside the q tile

    // ---- query fragments (B operand of S^T = K Q^T): lane holds row l16 of each 16-row block,
    //      head-dim chunk 32 ks + 8 g4
    bf16x8 qf[TQ][KS];
    int posq[TQ], wq_max[TQ], wq_min[TQ];
    bool row_ok[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        const int rloc = wrow0 + 16 * qb + l16;
        row_ok[qb] = rloc < q_n_rows;
        const int r = q_row_start + (row_ok[qb] ? rloc : q_n_rows - 1);
        const bf16_t *qp = p.q + b * p.qs_b + h * p.qs_h + (int64_t)(p.q_rowmap ? p.q_rowmap[r] : r) * p.qs_n + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *(const bf16x8 *)(qp + ks * 32);
        posq[qb] = p.pos_packed[r];
        const int sub = rg * TQ + qb;                  // 16-row granule of the q tile (wavefront-uniform)
        wq_max[qb] = __builtin_amdgcn_readfirstlane(sub < 16 ? qtp->sub_max[sub] : INT_MIN);
        wq_min[qb] = __builtin_amdgcn_readfirstlane(sub < 16 ? qtp->sub_min[sub] : INT_MAX);
    }

    int qlim[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) qlim[qb] = p.causal ? posq[qb] : INT_MAX - 1;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // wavefront-level position bounds; without a causal mask nothing is skipped or compared by position
    const int wq_hi = p.causal ? max(wq_max[0], wq_max[1]) : INT_MAX;
    const int wq_lo = p.causal ? min(wq_min[0], wq_min[1]) : INT_MAX;

    // ---- key/value tile range.  The tiles some query row of the workgroup can see (smallest key
    // position <= largest query position) form a prefix of the range: the tile list is ordered by
    // smallest position, over the whole sequence (fused) or inside each shard's range.
    const int t_begin = p.fused ? 0 : ((int_cptr)p.kv_shard_first)[kk];
    const int t_cap = p.fused ? p.n_kvtiles : ((int_cptr)p.kv_shard_first)[kk + 1];
    int t_end = t_cap;
    if (p.causal) {
        int n = 0;
        for (int base = t_begin; base < t_cap; base += 64) {
            const int t = base + lane;
            n += __popcll(__ballot(t < t_cap && p.kvtiles[t].pmin <= q_pmax));
        }
        t_end = t_begin + __builtin_amdgcn_readfirstlane(n);
    }
    // Tile metadata lives in scalar registers and is fetched ahead of its use (what the tile loads
    // need three tiles ahead, the block bounds one tile ahead), so the latency of the scalar loads
    // never sits on the critical path of a phase.
    struct TileMeta {
        int row_start, n_rows, index;                  // index: column block of V^T
    };
    struct TileBounds {
        int smin[4], smax[4];                          // position bounds of the four 16-key blocks
    };
    auto load_meta = [&](int t) {
        TileMeta m;
        const tile_cptr tp = kvtiles + t;
        m.row_start = tp->row_start; m.n_rows = tp->n_rows; m.index = tp->index;
        return m;
    };
    auto load_bounds = [&](int t) {
        TileBounds m;
        const tile_cptr tp = kvtiles + t;
#pragma unroll
        for (int kvb = 0; kvb < 4; ++kvb) { m.smin[kvb] = tp->sub_min[kvb]; m.smax[kvb] = tp->sub_max[kvb]; }
        return m;
    };

    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(p.k + b * p.ks_b + g * p.ks_h), 0, p.k_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(p.vt + b * p.vts_b + g * p.vts_h), 0, p.vt_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int32_t *>(p.pos_kv), 0, (uint32_t)p.N * 4, 0x00020000);

    // Direct-to-LDS loads of one tile.  K instruction i of this wavefront fills K rows
    // (wave*K_INSTR + i)*K_RPI ..: lane -> row lane/K_CPR, slot lane%K_CPR holding chunk slot^swz(row).
    // V^T instruction i fills V^T rows (wave*V_INSTR + i)*8 ..: lane -> row lane/8, slot lane%8.
    // The lane-dependent part of every offset is fixed for the whole kernel (32-bit: the launcher
    // checks that a (batch, kv head) slice stays below 2 GiB); a tile adds a scalar.
    uint32_t k_lane[K_INSTR], v_lane[V_INSTR];
    int k_rr[K_INSTR];
#pragma unroll
    for (int i = 0; i < K_INSTR; ++i) {
        const int rr = (wave * K_INSTR + i) * K_RPI + lane / K_CPR;
        const int slot = lane % K_CPR;
        const int c = D == 128 ? (slot ^ (rr & 15)) : (slot ^ ((rr >> 1) & 7));
        k_rr[i] = rr;
        k_lane[i] = (uint32_t)rr * (uint32_t)(p.ks_n * 2) + c * 16;
    }
#pragma unroll
    for (int i = 0; i < V_INSTR; ++i) {
        const int rr = (wave * V_INSTR + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((rr >> 1) & 7);
        v_lane[i] = (uint32_t)rr * (uint32_t)(p.npad * 2) + c * 16;
    }
    auto issue_loads = [&](const TileMeta &tm, int stage) {
        unsigned char *sk = smem + stage * STAGE;
        unsigned char *sv = sk + K_BYTES;
        const uint32_t k_tile = (uint32_t)tm.row_start * (uint32_t)(p.ks_n * 2);   // K is in packed row order here
        const uint32_t v_tile = (uint32_t)tm.index * (KV_TILE * 2);
#pragma unroll
        for (int i = 0; i < K_INSTR; ++i)
            load16_to_lds(rk, sk + (wave * K_INSTR + i) * K_RPI * K_ROW, k_rr[i] < tm.n_rows ? k_tile + k_lane[i] : OOB_OFF);
#pragma unroll
        for (int i = 0; i < V_INSTR; ++i)
            load16_to_lds(rv, sv + (wave * V_INSTR + i) * 8 * 128, v_tile + v_lane[i]);
        // every wavefront writes the same 64 positions: keeps the loads-per-tile count uniform
        load4_to_lds(rp, sv + V_BYTES, lane < tm.n_rows ? (uint32_t)(tm.row_start + lane) * 4 : OOB_OFF);
    };

    f32x4 oacc[TQ][DB];
    // m_run is the exponent offset in use (log2 units), m_top the true running maximum.  The offset
    // follows the maximum lazily: it moves only when some row's maximum has grown by more than
    // RESCALE_LOG2 since the offset was set, so exponentials stay below 2^RESCALE_LOG2 and the
    // rescaling of O and of the running sum is skipped for most tiles.  The results are the same
    // in exact arithmetic; m and e are referred to the true maximum on write-out.
    constexpr float RESCALE_LOG2 = 8.0f;
    float m_run[TQ], m_top[TQ], l_run[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        m_run[qb] = -INFINITY;
        m_top[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // operand read swizzles
    const int k_swz = D == 128 ? l16 : (l16 >> 1);
    const int v_swz = l16 >> 1;

    // ---- main loop, skewed schedule.  The 8 wavefronts form two groups of 4 (wavefronts w and w+4
    // share a SIMD).  Each visible tile i takes a matrix phase and a vector phase:
    //   X(i)  S^T(i) = K(i) Q^T  and  O^T += V^T(i-1) P^T(i-1)        (LDS reads + MFMAs)
    //   Y(i)  mask, row max, exponentials -> P(i); rescale O           (VALU only)
    // and there is one workgroup barrier per tile.  Between barriers i and i+1 group 0 runs X(i), Y(i)
    // and group 1 runs Y(i-1), X(i): on each SIMD one wavefront is in a matrix phase while the other is
    // in a vector phase, without a second barrier to enforce it.  The P V product trails by one tile,
    // so a matrix phase never waits for the exponentials of its own tile.
    // Tiles are NST = 4 stages deep in LDS.  The loads of tile i+2 are issued in X(i), i.e. after
    // barrier i, which every wavefront reaches only after its X(i-1): the stage they overwrite held
    // tile i-2, whose K was last read in X(i-2) and whose V^T in X(i-1).  Before barrier i+1 each
    // wavefront waits for its own loads of tile i+1, so the tile is complete when X(i+1) starts.
    constexpr int NST = 4;
    constexpr int LPT = K_INSTR + V_INSTR + 1;         // direct-to-LDS loads per tile per wavefront
    const int group = NWV == 8 ? wave >> 2 : 0;
    int t = t_begin;                                   // tile i
    TileMeta mt0 = {}, mt1 = {}, mt2 = {};             // tiles i, i+1, i+2
    if (t < t_end) mt0 = load_meta(t);
    if (t + 1 < t_end) mt1 = load_meta(t + 1);
    if (t + 2 < t_end) mt2 = load_meta(t + 2);
    TileBounds bd0 = {}, bd1 = {};                     // tiles i, i+1
    if (t < t_end) bd0 = load_bounds(t);
    if (t < t_end) issue_loads(mt0, 0);
    if (t + 1 < t_end) issue_loads(mt1, 1);
    if (t + 1 < t_end) phase_barrier<LPT, false>();    // barrier 0: tile 0 complete and visible
    else phase_barrier<0, false>();

    f32x4 sacc[TQ][4];                                 // S^T of the tile between its X and its Y
    bf16x8 pf[TQ][2];                                  // P^T operands of the tile whose P V product is pending
    int n_act = 0, maskm = 0, kn = KV_TILE;            // of the tile held in sacc
    int y_stage = 0;                                   // its stage
    int n_pv = 0;                                      // 32-key steps of the pending P V product that hold non-zero P

    auto pv_steps = [&](auto ns_tag, int stg) {
        constexpr int NS = decltype(ns_tag)::value;
        const unsigned char *pv = smem + stg * STAGE + K_BYTES + l16 * 128;
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) {
            const int cv = ((4 * s2 + g4) ^ v_swz) * 16;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 vf = *(const bf16x8 *)(pv + db * 16 * 128 + cv);
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    oacc[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qb][s2], oacc[qb][db], 0, 0, 0);
            }
        }
    };
    // S^T blocks: sacc[qb][kvb] = K[kvb] Q[qb]^T (16 keys x 16 queries) for the first NA blocks, zeros beyond
    auto qk_blocks = [&](auto na_tag, const unsigned char *sk) {
        constexpr int NA = decltype(na_tag)::value;
#pragma unroll
        for (int kvb = 0; kvb < 4; ++kvb) {
            if (kvb >= NA) {
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb) sacc[qb][kvb] = zero4;
                continue;
            }
            const unsigned char *kp = sk + (kvb * 16 + l16) * K_ROW;
            bf16x8 kf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks] = *(const bf16x8 *)(kp + (((4 * ks + g4) ^ k_swz) * 16));
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    sacc[qb][kvb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[qb][ks],
                                                                            ks == 0 ? zero4 : sacc[qb][kvb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);         // keeps at most one block's operands in registers
        }
    };

    // Both products of a full tile (all four key blocks visible, a full P pending), interleaved so that
    // the LDS latency of one product's operand reads is covered by the other's MFMAs: per key block b,
    // V^T reads of quarter b of O^T += V^T P^T, the 8 MFMAs of S^T block b (its K operands were read a
    // step earlier), K reads of block b+1, the 8 MFMAs of that quarter.
    auto x_full_tile = [&](int stg, const unsigned char *sk) {
        const unsigned char *pv = smem + stg * STAGE + K_BYTES + l16 * 128;
        bf16x8 kf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = *(const bf16x8 *)(sk + l16 * K_ROW + (((4 * ks + g4) ^ k_swz) * 16));
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            constexpr int QD = DB / 4;                     // d-blocks per quarter of the P V product
            const int s2 = b >> 1, db0 = (b & 1) * 2 * QD;
            const int cv = ((4 * s2 + g4) ^ v_swz) * 16;
            bf16x8 vf[2 * QD];
#pragma unroll
            for (int q = 0; q < 2 * QD; ++q) vf[q] = *(const bf16x8 *)(pv + (db0 + q) * 16 * 128 + cv);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    sacc[qb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[qb][ks],
                                                                          ks == 0 ? zero4 : sacc[qb][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (b + 1 < 4) {
                const unsigned char *kp = sk + ((b + 1) * 16 + l16) * K_ROW;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf[ks] = *(const bf16x8 *)(kp + (((4 * ks + g4) ^ k_swz) * 16));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 2 * QD; ++q)
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
                    oacc[qb][db0 + q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[q], pf[qb][s2], oacc[qb][db0 + q], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ================= X(i): matrix phase
    auto matrix_phase = [&](int i) {
        const int stage = i % NST;
        const unsigned char *sk = smem + stage * STAGE;
        y_stage = stage;
        if (t + 2 < t_end) issue_loads(mt2, (i + 2) % NST);
        // The SIMD's other wavefront is in its vector phase: let this one's MFMAs and operand reads win the
        // issue arbitration, so the matrix pipe is fed first and the softmax arithmetic fills the gaps.
        __builtin_amdgcn_s_setprio(3);
        // O^T += V^T(i-1) P^T(i-1).  Step s covers keys 32s..32s+31; k-slot (g4, j) of both operands is
        // key 32s + 16(j/4) + 4 g4 + j%4, i.e. accumulator register j%4 of block 2s + j/4.
        const int prev_stage = (i + NST - 1) % NST;
        // per 16-key block: can this wavefront skip it / does it need the element-wise compare
        kn = mt0.n_rows;
        int skipm = 0;
        maskm = 0;
#pragma unroll
        for (int kvb = 0; kvb < 4; ++kvb) {
            const int kmin = bd0.smin[kvb], kmax = bd0.smax[kvb];
            skipm |= (int)((kvb * 16 >= kn) | (kmin > wq_hi)) << kvb;
            maskm |= (int)((kvb * 16 + 16 > kn) | (kmax > wq_lo)) << kvb;
        }
        // With positions ascending along a tile the blocks this wavefront cannot see are the trailing
        // ones: blocks [0, n_act) are computed (for other position orders one below n_act that could
        // have been skipped is cut by the element-wise compare instead), blocks [n_act, 4) contribute
        // exact zeros to P.
        const int n_act_new = (~skipm & 15) ? 32 - __builtin_clz(~skipm & 15) : 0;
        maskm &= (1 << n_act_new) - 1;                 // blocks that are not computed need no compare
        if (n_pv == 2 && n_act_new == 4) {
            x_full_tile(prev_stage, sk);
        } else {
            if (n_pv == 2) pv_steps(std::integral_constant<int, 2>(), prev_stage);
            else if (n_pv == 1) pv_steps(std::integral_constant<int, 1>(), prev_stage);
            __builtin_amdgcn_sched_barrier(0);
            switch (n_act_new) {
                case 4: qk_blocks(std::integral_constant<int, 4>(), sk); break;
                case 3: qk_blocks(std::integral_constant<int, 3>(), sk); break;
                case 2: qk_blocks(std::integral_constant<int, 2>(), sk); break;
                case 1: qk_blocks(std::integral_constant<int, 1>(), sk); break;
                default: qk_blocks(std::integral_constant<int, 0>(), sk);
            }
        }
        n_act = n_act_new;
        __builtin_amdgcn_s_setprio(0);
    };

    // ================= Y(i): vector phase on the tile held in sacc
    auto vector_phase = [&]() {
        if (maskm) {                                   // some visible block needs the element-wise compare
            // Key positions of this lane's accumulator rows (keys 16 kvb + 4 g4 + 0..3), from the tile's
            // stage.  Read in assembly, wait included: the compiler would otherwise order a typed LDS read
            // after every tile load in flight, and the registers are needed only from here on.
            typedef __attribute__((ext_vector_type(4))) int i32x4;
            i32x4 pkv[4];
            {
                const uint32_t pa = (uint32_t)(uintptr_t)(lds_void *)(smem + y_stage * STAGE + K_BYTES + V_BYTES) + 16 * g4;
                asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:64\n\tds_read_b128 %2, %4 offset:128\n\t"
                             "ds_read_b128 %3, %4 offset:192\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(pkv[0]), "=&v"(pkv[1]), "=&v"(pkv[2]), "=&v"(pkv[3])
                             : "v"(pa)
                             : "memory");
            }
            int pk[4][4];
#pragma unroll
            for (int kvb = 0; kvb < 4; ++kvb)
#pragma unroll
                for (int r = 0; r < 4; ++r) pk[kvb][r] = pkv[kvb][r];
            if (kn < KV_TILE) {                            // ragged tile: keys past its end are never visible
#pragma unroll
                for (int kvb = 0; kvb < 4; ++kvb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (kvb * 16 + 4 * g4 + r >= kn) pk[kvb][r] = INT_MAX;
            }
            // mask.  sacc[qb][kvb][r]: key 16 kvb + 4 g4 + r, query l16.  With no causal mask the limit is
            // INT_MAX - 1, so only the keys past a ragged tile's end (position INT_MAX) are cut.
#pragma unroll
            for (int kvb = 0; kvb < 4; ++kvb) {
                if (kvb >= n_act || !(maskm & (1 << kvb))) continue;
#pragma unroll
                for (int qb = 0; qb < TQ; ++qb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (pk[kvb][r] > qlim[qb]) sacc[qb][kvb][r] = -INFINITY;
            }
        }
        // row statistics, exponentials, rescale of the running output (Algorithm 4's n, w, o online)
#pragma unroll
        for (int qb = 0; qb < TQ; ++qb) {
            float mx = -INFINITY;
#pragma unroll
            for (int kvb = 0; kvb < 4; ++kvb)
                if (kvb < n_act)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mx = fmaxf(mx, sacc[qb][kvb][r]);
            mx = xor_max_16_32(mx) * p.scale_log2;
            m_top[qb] = fmaxf(m_top[qb], mx);
            if (__builtin_amdgcn_readfirstlane(__any(mx > m_run[qb] + RESCALE_LOG2))) {
                const float m_new = fmaxf(m_run[qb], mx);
                const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - ((m_new == -INFINITY) ? 0.f : m_new));
                m_run[qb] = m_new;
                l_run[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db) oacc[qb][db] *= alpha;
            }
            const float m_sub = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
            float psum = 0.f;
#pragma unroll
            for (int kvb = 0; kvb < 4; ++kvb) {
                if (kvb >= n_act) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kvb][r], p.scale_log2, -m_sub));
                    sacc[qb][kvb][r] = pv;
                    psum += pv;
                }
            }
            l_run[qb] += psum;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    pf[qb][s2][j] = (bf16_t)sacc[qb][2 * s2][j];
                    pf[qb][s2][4 + j] = (bf16_t)sacc[qb][2 * s2 + 1][j];
                }
        }
        n_pv = (n_act + 1) >> 1;
    };

    // one loop per group: the bodies differ only in the order of the two phases
#define ATTN_TILE_BODY(FIRST, SECOND)                                                             \
    for (; t < t_end; ++i, ++t) {                                                                 \
        TileMeta mt3 = mt2;                                                                       \
        if (t + 3 < t_end) mt3 = load_meta(t + 3);                                                \
        if (t + 1 < t_end) bd1 = load_bounds(t + 1);                                              \
        FIRST;                                                                                    \
        SECOND;                                                                                   \
        /* barrier i+1: own loads of tile i+1 landed (those of tile i+2, if any, stay in flight), */ \
        /* own operand reads of this phase returned */                                            \
        if (t + 2 < t_end) phase_barrier<LPT, true>();                                            \
        else phase_barrier<0, true>();                                                            \
        mt0 = mt1; mt1 = mt2; mt2 = mt3;                                                          \
        bd0 = bd1;                                                                                \
    }
    int i = 0;
    if (group == 0) {
        ATTN_TILE_BODY(matrix_phase(i), vector_phase())            // X(i), Y(i)
    } else {
        ATTN_TILE_BODY(if (i > 0) vector_phase(), matrix_phase(i)) // Y(i-1), X(i)
        if (i > 0) vector_phase();                                 // Y of the last tile
    }
#undef ATTN_TILE_BODY
    // the trailing P V product of the last tile
    {
        const int prev_stage = (i + NST - 1) % NST;
        if (n_pv == 2) pv_steps(std::integral_constant<int, 2>(), prev_stage);
        else if (n_pv == 1) pv_steps(std::integral_constant<int, 1>(), prev_stage);
    }

    // ---- write-out.  oacc[qb][db][r]: query row 16qb + l16, column 16db + 4 g4 + r.
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        const float l_tot = xor_sum_16_32(l_run[qb]);
        if (!row_ok[qb]) continue;
        const int r = q_row_start + wrow0 + 16 * qb + l16;
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        if (p.fused) {
            bf16_t *op = p.o + ((int64_t)b * p.N + (p.o_rowmap ? p.o_rowmap[r] : r)) * p.o_ld + (int64_t)h * D + 4 * g4;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const f32x4 v = oacc[qb][db] * inv;
                *(bf16x4 *)(op + 16 * db) = bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
            }
        } else {
            const int64_t me = (((int64_t)b * p.H + h) * p.S + kk) * p.N + r;
            // refer the sum and the unnormalised output to the true maximum
            const float corr = m_top[qb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run[qb] - m_top[qb]);
            if (g4 == 0) {
                p.m[me] = m_top[qb] * LN2;
                p.e[me] = l_tot * corr;
            }
            const float f = p.u_mode == CASCADE_U_NORMALISED ? inv : corr;
            float *up = p.u + ((((int64_t)b * p.S + kk) * p.H + h) * p.N + r) * D + 4 * g4;
#pragma unroll
            for (int db = 0; db < DB; ++db) *(f32x4 *)(up + 16 * db) = oacc[qb][db] * f;
        }
    }
}

static int32_t npad_of(const cascade_plan *p) { return std::max(1, plan_tiles(kv_plan(p), KV_TILE).count) * KV_TILE; }

// V^T (tile order, padded) followed by room for K gathered into packed order
static size_t vt_bytes_of(const cascade_plan *p, int32_t B, int32_t Hkv, int32_t d) {
    return align_up((size_t)B * Hkv * d * npad_of(p) * 2, 256);
}
size_t attn_bf16_workspace_bytes(const cascade_plan *p, int32_t B, int32_t Hkv, int32_t d) {
    return vt_bytes_of(p, B, Hkv, d) + align_up((size_t)B * Hkv * p->seq_len * d * 2, 256);
}

// split: fused mode only; 32-row query tiles for the fused kernel's split walk (see attn_bf16_fused.hip)
template <int D, int NWV>
static int32_t launch_attn_cfg(const cascade_plan *p, const AttnArgs &a, hipStream_t s, bool split = false) {
    const cascade_plan *kvp = kv_plan(p);                      // key/value shards (S); query tiles follow p (R)
    const int N = p->seq_len, S = kvp->n_shards;
    const int rep = a.H / a.Hkv;
    const int hpb = rep % 4 == 0 ? 4 : rep % 2 == 0 ? 2 : 1;
    const int rowgroups = NWV / hpb;
    const int granule = split ? 32 : 32 * rowgroups;           // 32 .. 256 query rows per workgroup
    const CascadeTileList &ql = plan_tiles(p, granule);
    const CascadeTileList &kl = plan_tiles(kvp, KV_TILE);
    const int npad = npad_of(p);
    if (ql.count == 0) return CASCADE_OK;

    bf16_t *vt = (bf16_t *)a.workspace;
    bf16_t *kp = a.kv_rowmap ? (bf16_t *)((unsigned char *)a.workspace + vt_bytes_of(p, a.B, a.Hkv, D)) : nullptr;
    {   // V^T in tile order and, where K is not in packed order, K gathered into it: one launch
        dim3 grid(kl.count, a.Hkv, a.B);
        hipLaunchKernelGGL(vtranspose_kernel<D>, grid, dim3(256), 0, s, (const bf16_t *)a.v, vt, a.ks_b, a.ks_h,
                           a.ks_n, npad, a.Hkv, kl.dev, a.kv_rowmap, (const bf16_t *)a.k, kp, N);
        CASCADE_HIP_TRY(hipGetLastError());
    }
    AttnBf16Params k;
    k.q = (const bf16_t *)a.q; k.k = (const bf16_t *)a.k; k.vt = vt;
    k.qs_b = a.qs_b; k.qs_h = a.qs_h; k.qs_n = a.qs_n; k.ks_b = a.ks_b; k.ks_h = a.ks_h; k.ks_n = a.ks_n;
    if (kp) { k.k = kp; k.ks_n = D; k.ks_h = (int64_t)N * D; k.ks_b = (int64_t)a.Hkv * N * D; }
    k.vts_b = (int64_t)a.Hkv * D * npad; k.vts_h = (int64_t)D * npad; k.npad = npad;
    const int64_t kb = ((int64_t)(N - 1) * k.ks_n + D) * 2, vb = (int64_t)D * npad * 2;
    if (kb >= (int64_t)OOB_OFF || vb >= (int64_t)OOB_OFF) return CASCADE_EUNSUPPORTED;
    k.k_bytes = (uint32_t)kb; k.vt_bytes = (uint32_t)vb;
    k.q_rowmap = a.q_rowmap;
    // Under a causal mask a tile's work grows with its largest position: longest tiles first, so that a
    // launch of several rounds does not end on a long workgroup.
    k.qtiles = a.mask_kind == CASCADE_MASK_CAUSAL ? ql.dev_by_pmax_desc : ql.dev; k.kvtiles = a.fused ? kl.dev_by_pmin : kl.dev_by_shard_pmin; k.kv_shard_first = kl.shard_first; k.n_kvtiles = kl.count;
    k.pos_packed = p->pos_packed_d; k.pos_kv = kvp->pos_packed_d; k.pos_kv_padded = kl.pos_padded;
    k.B = a.B; k.H = a.H; k.Hkv = a.Hkv; k.N = N; k.S = S;
    k.scale_log2 = a.scale * LOG2E;
    k.causal = a.mask_kind == CASCADE_MASK_CAUSAL; k.fused = a.fused; k.u_mode = a.u_mode;
    k.m = a.m; k.e = a.e; k.u = a.u; k.o = (bf16_t *)a.o; k.o_ld = a.o_ld; k.o_rowmap = a.o_rowmap;
    k.hpb = hpb;

    constexpr int lds = 4 * (KV_TILE * D * 2 + D * 128 + KV_TILE * 4);
    auto kern = attn_bf16_kernel<D, NWV>;
    static std::atomic<uint64_t> lds_ready{0};
    CASCADE_HIP_TRY(ensure_dynamic_lds((const void *)kern, lds, lds_ready));
    const int64_t gy = (int64_t)a.B * a.Hkv * (rep / hpb);
    if (gy * ql.count > INT32_MAX || S > 65535) return CASCADE_EUNSUPPORTED;
    k.gy = (int32_t)gy;
    for (k.hpb_log2 = 0; (1 << k.hpb_log2) < hpb; ++k.hpb_log2) {}
    k.rep = rep; k.hblocks = rep / hpb; k.heads = a.Hkv * k.hblocks;
    k.gy_magic = div_magic((uint32_t)gy); k.heads_magic = div_magic((uint32_t)k.heads); k.hblocks_magic = div_magic((uint32_t)k.hblocks);
    // fused mode with full-size query tiles: the software-pipelined kernel (same tiles, same parameters; its mask
    // forms "query position - key position" in 32 bits: positions below 2^30 in magnitude)
    if (a.fused && NWV == 8 && p->max_abs_pos < (1 << 30) && kvp->max_abs_pos < (1 << 30)) {
        bool all_visible = a.mask_kind != CASCADE_MASK_CAUSAL;
        for (int j = 0; j < kvp->n_shards && all_visible; ++j)
            all_visible = (kvp->offsets_h[j + 1] - kvp->offsets_h[j]) % KV_TILE == 0;
        if (!div_magic_covers((uint64_t)gy * ql.count, (uint32_t)gy)) return CASCADE_EUNSUPPORTED;
        return launch_attn_fused(k, D, ql.count, all_visible, split, s);
    }
    if (split) return CASCADE_EINVAL;
    dim3 grid((unsigned)(gy * ql.count), 1, a.fused ? 1 : S);
    hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), lds, s, k);
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
    // FUSED mode under a causal mask, launches of more than one round of workgroups: walk queries and keys in
    // ascending position (the plan's one-shard view; q, k, v and o rows are reached through its row map, K and
    // V^T are gathered in that order).  Tiles of a shard of scattered tokens span a large part of the sequence,
    // so that most (query tile, key tile) pairs are partly masked and a third to a half of the products of the
    // shard-ordered walk are thrown away; in position order only the diagonal tiles are.  The result is the same:
    // the merge over key/value shards does not depend on how the keys are grouped.  A launch of a single round
    // gains nothing (its duration is that of the workgroup with the last query rows, which sees every tile either
    // way) and keeps the shard order, which needs no gather of K.
    if (a.fused && a.mask_kind == CASCADE_MASK_CAUSAL && p->sorted && !a.q_rowmap && !a.o_rowmap &&
        p->max_abs_pos < (1 << 30)) {
        const int rep = a.H / a.Hkv;
        const int hpb = rep % 4 == 0 ? 4 : rep % 2 == 0 ? 2 : 1;
        const int granule = 32 * (8 / hpb);
        const int64_t wgs = (int64_t)a.B * a.Hkv * (rep / hpb) * ((p->seq_len + granule - 1) / granule);
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 256;
        // A launch of a single round: with four heads per workgroup the split walk (32-row query tiles, the two
        // wavefront groups of a workgroup take every other key/value tile) doubles the workgroups and halves the
        // longest walk; it needs the position order for its tile counts to be even.
        const bool split = wgs <= cus && hpb == 4 && p->seq_len >= 4 * KV_TILE;
        if ((wgs > cus && p->seq_len > 32 * (4 / hpb)) || split) {
            AttnArgs b = a;
            b.q_rowmap = b.o_rowmap = b.kv_rowmap = p->sorted_to_row_d;
            if (a.d == 128) return launch_attn_cfg<128, 8>(p->sorted, b, s, split);
            return launch_attn_cfg<64, 8>(p->sorted, b, s, split);
        }
    }
    // 8 wavefronts cover 256 / hpb query rows of a shard; when no shard of the plan has more than half of that,
    // four of them would never have rows: use the 4-wavefront workgroup
    const int rep = a.H / a.Hkv;
    const int hpb = rep % 4 == 0 ? 4 : rep % 2 == 0 ? 2 : 1;
    int max_shard = 0;
    for (int j = 0; j < p->n_shards; ++j) max_shard = std::max(max_shard, p->offsets_h[j + 1] - p->offsets_h[j]);
    const bool half = max_shard <= 32 * (4 / hpb);
    if (a.d == 128) return half ? launch_attn_cfg<128, 4>(p, a, s) : launch_attn_cfg<128, 8>(p, a, s);
    return half ? launch_attn_cfg<64, 4>(p, a, s) : launch_attn_cfg<64, 8>(p, a, s);
}
