// Fused bf16 attention for the layer path: the attention-pass of every (query shard, key/value shard) pair
// (Algorithm 3) with the post-pass merge (the running n, w, o of Algorithm 4) kept in registers while the
// key/value tiles of all shards are walked.  Software-pipelined inside each wavefront.
//
// Work split and data layout are those of the partial-attention kernel (attn_bf16.hip): a workgroup of 8
// wavefronts, two per SIMD, owns one tile of packed query rows for up to 4 query heads sharing a key/value
// head; a wavefront owns 32 query rows of one head; S^T = K Q^T so a lane holds one query row; O^T = V^T P^T
// with the exponentials going from the accumulator layout straight into the B operand; 64-key tiles of K,
// V^T (key-permuted) and key positions go from L2/HBM straight into LDS, four stages, swizzled rows.
//
// What is different.  The three independent streams of work of a step are interleaved by hand inside the
// wavefront, instruction by instruction:
//
//   step k (half tile = 32 keys):   MFMA   S^T(k)   = -m + K(k) Q'^T      (scores of half tile k: log2 units, offset taken off)
//                                   MFMA   O^T     += V^T(k-2) P^T(k-2)   (trailing by two half tiles)
//                                   MFMA   l       += 1 P^T(k-2)          (row sums: the same product against ones)
//                                   VALU   P(k-1)   = exp2(S(k-1))
//                                   VALU   lane maximum of S(k), and its mask where the tile needs one
//
// Q' is Q scaled by scale * log2(e) when the wavefront loads its query fragments (once; one more rounding of q
// to bf16), and the score product starts from minus the row's exponent offset m instead of zero (a lane's four
// accumulator values belong to one query, so the initial value is one register quad per query block): the
// exponential then needs no multiply-add in front of it, one vector instruction less per score (C4 attention -5 %).
// When an offset moves, the scores of the step just done, which were taken against the old one, are shifted.
//
// Measured on MI355X (one wavefront, loops of MFMAs with vector instructions behind each): a 16x16x32 MFMA
// holds the matrix pipe for 16 cycles but the wavefront's issue for 8, a vector instruction takes 4 (an
// exponential ~9), so two vector instructions per MFMA are free and every further one costs its full time;
// a taken branch costs ~50 cycles (the kernel is issue-bound: one instruction stream per wavefront, and the
// scalar, LDS and vector instructions of a wavefront only overlap with those of the SIMD's other wavefront).
// Hence: the MFMAs are inline assembly in a fixed order with the vector arithmetic cut into chunks of a few
// instructions between them (a scheduling barrier after every group keeps the compiler from regrouping them);
// a step is straight-line code but for one branch around the mask; the row sums and the rescaling bookkeeping
// cost no vector instructions; operand fragments are read from LDS RD fragments ahead
// through a register ring, across step boundaries; tile loads are requested two tile periods ahead and the
// barrier waits with a counted vmcnt, not for the youngest requests.
// (Tried and measured slower: one wavefront per SIMD with 64 query rows, i.e. half the LDS reads per MFMA
// and 512 registers - without a second wavefront nothing overlaps its scalar instructions and waits.)
//
// Rules this file has to keep, because the compiler does not see the MFMAs:
//  * nothing but the MFMA statements may touch the accumulators (O^T, row sums) inside the tile loop; a
//    compiler-visible use there makes it copy them between register files right behind an MFMA that is still
//    in flight.  That is why a late move of an exponent offset restarts the pass instead of rescaling.
//  * a register an MFMA reads must not be written by a vector instruction directly in front of it (the
//    hardware needs wait states the compiler only inserts for MFMAs it knows): constants fed to MFMAs are
//    made opaque so that they are not rebuilt in place; the build scans the ISA for both conditions.
//  * every MFMA statement appears once in the loop (two copies make the register allocator shuffle the
//    accumulators between them), so "masked or not" is a kernel parameter, not a choice per tile.
//
// The exponent offset m of a row is an integer (the ceiling of the running maximum in log2 units) that is
// set by the row's first visible score and moves only when a later maximum exceeds it by more than 2^40.
#include <climits>
#include <cstdlib>
#include <type_traits>
#include <utility>
#include "attn_bf16.h"

namespace {

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

// S^T accumulators live in vector registers (the softmax reads them), query fragments in accumulation
// registers; O^T accumulators in accumulation registers.
__device__ __forceinline__ void mfma_s_first(f32x4 &c, const bf16x8 &k, const bf16x8 &q, const f32x4 &init) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(k), "a"(q), "v"(init));
}
__device__ __forceinline__ void mfma_s(f32x4 &c, const bf16x8 &k, const bf16x8 &q) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_o(f32x4 &c, const bf16x8 &vt, const bf16x8 &pt) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(vt), "v"(pt));
}
// The compiler does not see those MFMAs: before anything else touches their results, let the last
// ones leave the matrix pipeline.
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }
__device__ __forceinline__ void fence() { __builtin_amdgcn_sched_barrier(0); }

}   // namespace

// TQ: 16-row query blocks per wavefront (2: 32 rows, 8 wavefronts; 4: 64 rows, 4 wavefronts).  MASKED: the kernel
// holds the code that compares a score with its key's position (causal plans, plans with ragged key/value tiles);
// false only when every key of every tile is visible to every query.  A kernel parameter: a second copy of the
// MFMA statements inside the loop makes the register allocator shuffle the accumulators between the copies.
// Inside a MASKED kernel the comparisons of a step (2 instructions per score, a third of the step's vector
// arithmetic) sit behind one wavefront-uniform branch and run only for tiles that hold a key some query of the
// wavefront cannot see or that are padded: with the walk in position order that is the last one or two tiles
// (C4 / C5 attention -6 %).
// SPLIT (TQ = 2, MASKED, four heads per workgroup): the two wavefront groups take the same 32 query rows and every
// other key/value tile each, and their running (offset, row sum, output) are merged through LDS at the end.  For
// launches of a single round of workgroups: a query tile's walk is then half as long and there are twice as many
// workgroups, so that the CUs with early (short) query tiles take a second one instead of idling.
template <int D, int TQ, bool MASKED, bool SPLIT = false>
__global__ __launch_bounds__(1024 / TQ) void attn_fused_kernel(AttnBf16Params p) {
    static_assert(!SPLIT || (TQ == 2 && MASKED), "the split walk exists for the masked 8-wavefront kernel");
    constexpr int KS = D / 32;                         // k-steps of the score product
    constexpr int DB = D / 16;                         // 16-row blocks of O^T
    constexpr int K_ROW = D * 2;                       // bytes per K row in LDS
    constexpr int K_RPI = 1024 / K_ROW;                // K rows filled by one direct-to-LDS instruction
    constexpr int K_CPR = K_ROW / 16;
    constexpr int K_BYTES = KV_TILE * K_ROW, V_BYTES = D * 128;
    constexpr int STAGE = K_BYTES + V_BYTES + KV_TILE * 4;
    constexpr int NWV = 16 / TQ, NST = 4;              // 4 wavefronts (one per SIMD) or 8 (two per SIMD)
    constexpr int K_INSTR = KV_TILE / K_RPI / NWV, V_INSTR = D / 8 / NWV;
    constexpr int NQF = 2 * KS, NVF = DB;              // operand fragments per step: K (2 key blocks), V^T
    constexpr float RESCALE_LOG2 = 40.0f;              // exponentials stay below 2^40

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g4 = lane >> 4;
    // workgroup -> (query tile, batch, kv head, head block): multiplications by reciprocals the launcher made
    // (a division by a kernel argument is ~25 scalar instructions, and there were seven in front of the first load)
    const int hpb_log2 = SPLIT ? 2 : p.hpb_log2, hpb = 1 << hpb_log2;
    const int hsel = wave & (hpb - 1), rg = wave >> hpb_log2;
    const int rep = p.rep, hblocks = p.hblocks;
    const int q_tile = (int)div_by_magic(blockIdx.x, p.gy_magic), by = (int)blockIdx.x - q_tile * p.gy;
    const int b = (int)div_by_magic((uint32_t)by, p.heads_magic), gh = by - b * p.heads;
    const int g = (int)div_by_magic((uint32_t)gh, p.hblocks_magic);
    const int h = g * rep + (gh - g * hblocks) * hpb + hsel;

    const tile_cptr kvtiles = (tile_cptr)p.kvtiles;
    const tile_cptr qtp = (tile_cptr)p.qtiles + q_tile;
    const int q_row_start = qtp->row_start, q_n_rows = qtp->n_rows, q_pmax = qtp->pmax;
    const int wrow0 = SPLIT ? 0 : rg * 16 * TQ;       // SPLIT: both wavefront groups hold the query tile's 32 rows

    // ---- Everything below up to the first barrier is one chain of dependent accesses per workgroup (tile entry ->
    // row map -> query rows; tile entry -> visible tiles -> their entries -> K rows), so the requests of a level go
    // out together and nothing is waited for in between: rows and limits first, then the tile list's smallest
    // positions, then the query rows.
    int qlim[TQ], q_src[TQ];
    bool row_ok[TQ];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        const int rloc = wrow0 + 16 * qb + l16;
        row_ok[qb] = rloc < q_n_rows;
        const int r = q_row_start + (row_ok[qb] ? rloc : q_n_rows - 1);
        q_src[qb] = p.q_rowmap ? p.q_rowmap[r] : r;
        // without a mask: the largest position the launcher accepts, so that only the padding of ragged tiles
        // (position 2^30) is cut; every position is below 2^30 in magnitude
        qlim[qb] = p.causal ? p.pos_packed[r] : (1 << 30) - 1;
    }
    // visible key/value tiles: a prefix of the list ordered by smallest position; four groups of 64 entries a time
    constexpr int VIS = 4;
    int pm_first[VIS];
    if (p.causal) {
#pragma unroll
        for (int c = 0; c < VIS; ++c) {
            const int t = 64 * c + lane;
            pm_first[c] = t < p.n_kvtiles ? p.kvtiles[t].pmin : INT_MAX;
        }
    }

    // ---- query fragments (B operand of S^T = K Q^T): lane holds row l16 of each 16-row block, head-dim
    //      chunk 32 ks + 8 g4
    bf16x8 q_raw[TQ][KS];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        const bf16_t *qp = p.q + b * p.qs_b + h * p.qs_h + (int64_t)q_src[qb] * p.qs_n + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) q_raw[qb][ks] = *(const bf16x8 *)(qp + ks * 32);
    }

    int t_end = p.n_kvtiles;
    if (p.causal) {
        int n = 0;
#pragma unroll
        for (int c = 0; c < VIS; ++c) n += __popcll(__ballot(pm_first[c] <= q_pmax));
        for (int base = 64 * VIS; base < p.n_kvtiles; base += 64) {
            const int t = base + lane;
            n += __popcll(__ballot(t < p.n_kvtiles && p.kvtiles[t].pmin <= q_pmax));
        }
        t_end = __builtin_amdgcn_readfirstlane(n);
    }

    // The smallest limit of this wavefront's queries: a key/value tile whose largest position is not above it (and
    // that has no padding) is visible to every one of them, and its scores skip the mask.  From the tile entry's
    // 16-row minima (rows past the tile's end: INT_MAX; their lanes compute on the last row's limit and write nothing).
    int q_min = (1 << 30) - 1;
    if (p.causal) {
        q_min = qtp->sub_min[wrow0 / 16];
#pragma unroll
        for (int qb = 1; qb < TQ; ++qb) q_min = min(q_min, qtp->sub_min[wrow0 / 16 + qb]);
    }
    auto tile_needs_mask = [&](int tile_pmax, int tile_rows) { return tile_pmax > q_min || tile_rows < KV_TILE; };

    const int n_tiles = t_end;

    struct TileMeta {
        int row_start, n_rows, index, pmax;
    };
    auto load_meta = [&](int t) {
        TileMeta m;
        const tile_cptr tp = kvtiles + t;
        m.row_start = tp->row_start; m.n_rows = tp->n_rows; m.index = tp->index; m.pmax = tp->pmax;
        return m;
    };

    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(p.k + b * p.ks_b + g * p.ks_h), 0, p.k_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(p.vt + b * p.vts_b + g * p.vts_h), 0, p.vt_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int32_t *>(p.pos_kv_padded), 0, (uint32_t)p.n_kvtiles * KV_TILE * 4, 0x00020000);

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
    // K rows and key positions of a tile (K_INSTR + 1 loads per wavefront), V^T columns of a tile (V_INSTR loads)
    auto issue_k = [&](const TileMeta &tm, int stage) {          // stage: counted in STAGE bytes from smem
        unsigned char *sk = smem + stage * STAGE;
        const uint32_t k_tile = (uint32_t)tm.row_start * (uint32_t)(p.ks_n * 2);
#pragma unroll
        for (int i = 0; i < K_INSTR; ++i)
            load16_to_lds(rk, sk + (wave * K_INSTR + i) * K_RPI * K_ROW, k_rr[i] < tm.n_rows ? k_tile + k_lane[i] : OOB_OFF);
        // every wavefront writes the same 64 positions (2^30 past a ragged tile's end): keeps the
        // loads-per-batch count uniform
        load4_to_lds(rp, sk + K_BYTES + V_BYTES, (uint32_t)(tm.index * KV_TILE + lane) * 4);
    };
    auto issue_v = [&](const TileMeta &tm, int stage) {
        unsigned char *sv = smem + stage * STAGE + K_BYTES;
        const uint32_t v_tile = (uint32_t)tm.index * (KV_TILE * 2);
#pragma unroll
        for (int i = 0; i < V_INSTR; ++i)
            load16_to_lds(rv, sv + (wave * V_INSTR + i) * 8 * 128, v_tile + v_lane[i]);
    };

    // ---- the first tiles are requested here, ahead of the wait for the query rows.  The four entries are read
    // whatever the number of visible tiles (the index is clamped), so that they do not wait for that number.
    TileMeta mt0, mt1, mt2, mt3;                       // tiles i .. i+3 (split walk: j and j + 1 of either group)
    auto first_tiles = [&]() {
        const TileMeta none = {0, 0, 0, INT_MAX};
        const int last = p.n_kvtiles - 1;
        const TileMeta a0 = load_meta(0), a1 = load_meta(min(1, last)), a2 = load_meta(min(2, last)), a3 = load_meta(min(3, last));
        mt0 = 0 < n_tiles ? a0 : none;
        mt1 = 1 < n_tiles ? a1 : none;
        mt2 = 2 < n_tiles ? a2 : none;
        mt3 = 3 < n_tiles ? a3 : none;
        if constexpr (SPLIT) {                         // tiles 0 and 1 are the first of the two wavefront groups
            if (0 < n_tiles) issue_k(mt0, 0);
            if (1 < n_tiles) issue_k(mt1, 2);
        } else {
            if (0 < n_tiles) { issue_k(mt0, 0); issue_v(mt0, 0); }
            if (1 < n_tiles) { issue_k(mt1, 1); issue_v(mt1, 1); }
            if (2 < n_tiles) issue_k(mt2, 2);
        }
    };
    first_tiles();

    bf16x8 Q[TQ][KS];
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // scaled by scale * log2(e) here, once, so that the score product comes out in log2 units
#pragma unroll
            for (int x = 0; x < 8; ++x) Q[qb][ks][x] = (bf16_t)((float)q_raw[qb][ks][x] * p.scale_log2);
            // (in its accumulation registers here and now, not by moves right in front of the first MFMA that reads it)
            asm volatile("" : "+a"(Q[qb][ks]));
        }

    // ---- state
    f32x4 O[TQ][DB];                                   // accumulation registers
    f32x4 L[TQ];                                       // row sums of the exponentials, accumulated by the matrix pipe
    f32x4 S[2][TQ][2];                                 // scores of a half tile: [buffer][query block][key block]
    u32x4 P[2][TQ];                                    // exponentials of a half tile (8 bf16), B operand layout
    constexpr int RD = (D == 128 && !SPLIT ? 7 : 3);   // operand fragments read ahead of their use
    constexpr int RING = RD + 1;
    static_assert((NQF + NVF) % RING == 0, "the ring position of a step's first fragment must not move");
    bf16x8 ring[RING];                                 // operand fragments in flight
    float m_run[TQ], m_thr[TQ], lmax[TQ];
    f32x4 s_init[TQ];                                  // minus the row's exponent offset: the score product starts from it
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        // the threshold starts at the most negative finite value: any finite score passes it, -inf does not,
        // and "score - threshold" is never inf - inf
        m_run[qb] = -INFINITY; m_thr[qb] = -3.0e38f; lmax[qb] = -INFINITY;
        s_init[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // A block of ones as A operand turns the output product into the row sums.  The value is made opaque so
    // that it stays in four registers: rebuilt by moves right in front of an MFMA the compiler does not see,
    // it would be read before the moves have landed.
    bf16x8 ones = {(bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f, (bf16_t)1.f};
    asm volatile("" : "+v"(ones));
    const int k_swz = D == 128 ? l16 : (l16 >> 1);
    const int v_swz = l16 >> 1;
    const int kf_lane = l16 * K_ROW, vf_lane = l16 * 128;

    // Fragment f of a step whose score product reads half X of the K tile in stage qs and whose output
    // product reads half X of the V^T tile in stage vs: the K fragments come first, k-step by k-step with the
    // two key blocks alternating (an accumulator then recurs every 2 TQ MFMAs instead of every TQ: 1-2 % faster).
    // (Cutting the vector arithmetic into pieces of 3-5 instructions, one behind every MFMA, instead of chunks of
    // 10-12 behind every third or fourth, was measured 1-2 % slower: the SIMD's other wavefront fills the gaps.)
    // (qs: byte offset of the K tile's stage in LDS; vs: byte offset of the V^T tile itself)
    auto frag_ptr = [&](int qs, int vs, auto x_tag, int f) -> const unsigned char * {
        constexpr int X = decltype(x_tag)::value;
        if (f < NQF) {
            const int kvb = 2 * X + f % 2, ks = f / 2;
            return smem + qs + kvb * 16 * K_ROW + kf_lane + (((4 * ks + g4) ^ k_swz) * 16);
        }
        const int db = f - NQF;
        return smem + vs + db * 16 * 128 + vf_lane + (((4 * X + g4) ^ v_swz) * 16);
    };

    // ---- pieces of a step.  X = which half of their tiles the two products of the step read; the scores go
    // to S[X], the exponentials consumed by the output product are P[X]; the softmax turns S[1-X] into P[1-X].
    // Every chunk of vector arithmetic is bracketed by empty volatile assembly statements on its inputs and
    // results, which keeps the optimiser from hoisting or sinking it past the MFMAs it is placed between.
    typedef __attribute__((ext_vector_type(4))) int i32x4;

    // exponentials of the four scores of one (query block, key block) pair: chunk e = 2 qb + kb
    auto exp_chunk = [&](auto x_tag, auto e_tag) {
        constexpr int X = decltype(x_tag)::value, e = decltype(e_tag)::value;
        constexpr int qb = e / 2, kb = e % 2;
        const f32x4 sv = S[1 - X][qb][kb];
        const float p0 = __builtin_amdgcn_exp2f(sv[0]);    // the scores carry scale and offset already
        const float p1 = __builtin_amdgcn_exp2f(sv[1]);
        const float p2 = __builtin_amdgcn_exp2f(sv[2]);
        const float p3 = __builtin_amdgcn_exp2f(sv[3]);
        uint32_t w0 = __builtin_bit_cast(uint32_t, bf16x2{(bf16_t)p0, (bf16_t)p1});
        uint32_t w1 = __builtin_bit_cast(uint32_t, bf16x2{(bf16_t)p2, (bf16_t)p3});
        asm volatile("" : "+v"(w0), "+v"(w1));
        P[1 - X][qb][2 * kb] = w0;
        P[1 - X][qb][2 * kb + 1] = w1;
    };
    // mask of the four scores of one (query block, key block) pair of S[X]: a score whose key position is above
    // the query's becomes -inf: a compare and a select per score (measured 1-1.5 % faster over the kernel than
    // the branch-free form without a condition register: sign of limit - position inserted over the bits of
    // +inf, then a minimum, three instructions).
    auto mask_chunk = [&](auto x_tag, auto qb_tag, auto kb_tag, const i32x4 (&pk)[2]) {
        constexpr int X = decltype(x_tag)::value, qb = decltype(qb_tag)::value, kb = decltype(kb_tag)::value;
        f32x4 sv = S[X][qb][kb];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            sv[r] = qlim[qb] >= pk[kb][r] ? sv[r] : -INFINITY;
        }
        asm volatile("" : "+v"(sv));
        S[X][qb][kb] = sv;
    };
    // this lane's maximum over its 8 scores of query block qb of S[X] (log2 units); flagv collects by how much
    // a maximum is above its row's threshold
    auto max_chunk = [&](auto x_tag, auto qb_tag, float &flagv) {
        constexpr int X = decltype(x_tag)::value, qb = decltype(qb_tag)::value;
        const f32x4 a = S[X][qb][0], c = S[X][qb][1];
        // a chain of three-operand maxima: 4 instructions for the 8 scores (a balanced tree of pairs takes 6-7)
        float mx = fmaxf(fmaxf(a[0], a[1]), a[2]);
        mx = fmaxf(fmaxf(mx, a[3]), c[0]);
        mx = fmaxf(fmaxf(mx, c[1]), c[2]);
        mx = fmaxf(mx, c[3]) - s_init[qb][0];              // back to absolute log2 units
        float fl = fmaxf(flagv, mx - m_thr[qb]);
        asm volatile("" : "+v"(mx), "+v"(fl));
        lmax[qb] = mx;
        flagv = fl;
    };
    // key positions of this lane's accumulator rows (keys 16 kb + 4 g4 + 0..3 of half X) from the tile's stage
    // (2^30 for the keys past a ragged tile's end: never visible)
    auto read_positions = [&](auto x_tag, int qs, i32x4 (&pk)[2]) {
        constexpr int X = decltype(x_tag)::value;
        const unsigned char *pp = smem + qs + K_BYTES + V_BYTES + (32 * X + 4 * g4) * 4;
        pk[0] = *(const i32x4 *)pp;
        pk[1] = *(const i32x4 *)(pp + 64);
    };

    // ---- one step: scores of (qs, X) into S[X], output product of (vs, X) with P[X] (and the row sums: the
    // same product against a block of ones), exponentials of S[1-X] into P[1-X], then (MASKED, mask_on) the mask
    // and the lane maxima of the new scores.  Straight-line code but for the one branch around the mask: a taken
    // branch costs this kernel some fifty cycles.  On entry the ring holds the
    // first RD fragments; on exit those of the next step (half 1-X, stages nqs / nvs).  Returns whether some
    // maximum passed its row's threshold.
    // NEXT: whether the ring is refilled for the next step at all (false in front of a barrier that has yet to
    // confirm the next step's tiles: the caller then fills it behind the barrier).
    auto step = [&](auto x_tag, auto next_tag, int qs, int vs, int nqs, int nvs, bool mask_on) -> bool {
        constexpr bool NEXT = decltype(next_tag)::value;
        constexpr int X = decltype(x_tag)::value;
        constexpr int NF = NQF + NVF, QS = TQ * NQF, NS = TQ * NF + TQ;   // slots: scores, output, row sums
        constexpr int NE = 2 * TQ;                           // chunks of exponentials: one per (query block, key block) pair
        constexpr int NT = 3 * TQ;                           // chunks of the tail: per query block 2 of mask, 1 of maxima
        const std::integral_constant<int, 1 - X> nx;
        float flagv = 0.f;
        fence();
        auto after_slot = [&](auto s_tag) {
            constexpr int s = decltype(s_tag)::value;
            // exponentials: chunk e behind slot e * NS / NE + 1
            static_for<NE>([&](auto e_tag) {
                constexpr int e = decltype(e_tag)::value;
                if constexpr (e * NS / NE + 1 == s) exp_chunk(x_tag, e_tag);
            });
            // tail: chunk t behind slot QS + 2 + t * (NS - QS - 3) / NT (the scores are complete after slot QS - 1)
            static_for<NT>([&](auto t_tag) {
                constexpr int t = decltype(t_tag)::value;
                if constexpr (QS + 2 + t * (NS - QS - 3) / NT == s) {
                    constexpr int tq = t / 3, c = t % 3;
                    // The mask of the whole step sits in the first tail slot, behind one branch on a
                    // wavefront-uniform condition: in position order only the last one or two tiles of a walk hold
                    // a key some query of the wavefront cannot see, all others skip these 2 instructions per score.
                    if constexpr (t == 0 && MASKED) {
                        if (mask_on) {
                            i32x4 pk[2];
                            read_positions(x_tag, qs, pk);
                            static_for<2 * TQ>([&](auto m_tag) {
                                constexpr int m = decltype(m_tag)::value;
                                mask_chunk(x_tag, std::integral_constant<int, m / 2>{}, std::integral_constant<int, m % 2>{}, pk);
                            });
                        }
                    }
                    if constexpr (c == 2) max_chunk(x_tag, std::integral_constant<int, tq>{}, flagv);
                }
            });
            fence();
        };
        static_for<NF>([&](auto f_tag) {
            constexpr int f = decltype(f_tag)::value;
            // fragment f + RD of this step, or one of the first RD of the next
            if constexpr (f + RD < NF) ring[(f + RD) % RING] = *(const bf16x8 *)frag_ptr(qs, vs, x_tag, f + RD);
            else if constexpr (NEXT) ring[(f + RD) % RING] = *(const bf16x8 *)frag_ptr(nqs, nvs, nx, f + RD - NF);
            fence();
            static_for<TQ>([&](auto qb_tag) {
                constexpr int qb = decltype(qb_tag)::value;
                if constexpr (f < NQF) {
                    constexpr int kb = f % 2, ks = f / 2;
                    if constexpr (ks == 0) mfma_s_first(S[X][qb][kb], ring[f % RING], Q[qb][ks], s_init[qb]);
                    else mfma_s(S[X][qb][kb], ring[f % RING], Q[qb][ks]);
                } else {
                    mfma_o(O[qb][f - NQF], ring[f % RING], __builtin_bit_cast(bf16x8, P[X][qb]));
                }
                after_slot(std::integral_constant<int, TQ * f + qb>{});
            });
        });
        static_for<TQ>([&](auto qb_tag) {
            constexpr int qb = decltype(qb_tag)::value;
            mfma_o(L[qb], ones, __builtin_bit_cast(bf16x8, P[X][qb]));
            after_slot(std::integral_constant<int, TQ * NF + qb>{});
        });
        return __builtin_amdgcn_readfirstlane(__any(flagv > 0.f));
    };

    // ---- between steps.  A maximum that passed its row's threshold moves the row's exponent offset to the
    // ceiling of that maximum.  For a row without a maximum so far this is free (its exponentials were all
    // zero).  For a row that already has contributions the accumulators would have to be rescaled; nothing
    // but the MFMAs may touch them inside the loop (the compiler does not see those MFMAs and would move
    // accumulators around them), so that case, which needs a score 2^RESCALE_LOG2 times above everything
    // the row has seen before, abandons the pass instead: the offset moves, the pass runs to its end on
    // values nobody uses, and the whole workgroup starts over with the larger offsets.
    bool redo = false;
    auto between_steps = [&](auto x_tag, bool need) {
        constexpr int X = decltype(x_tag)::value;
        if (__builtin_expect(need, 0)) {
#pragma unroll
            for (int qb = 0; qb < TQ; ++qb) {
                const float rowmax = xor_max_16_32(lmax[qb]);
                const bool grow = rowmax > m_thr[qb];
                const float m_new = grow ? ceilf(rowmax) : m_run[qb];
                if (__builtin_amdgcn_readfirstlane(__any(grow && m_run[qb] != -INFINITY))) redo = true;
                m_run[qb] = m_new;
                m_thr[qb] = m_new == -INFINITY ? -3.0e38f : m_new + RESCALE_LOG2;
                const float nm_new = m_new == -INFINITY ? 0.f : -m_new;
                // the scores of the step just done were computed against the old offset
                const float delta = nm_new - s_init[qb][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) S[X][qb][kb] += f32x4{delta, delta, delta, delta};
                s_init[qb] = f32x4{nm_new, nm_new, nm_new, nm_new};
            }
        }
        fence();
    };

    // ---- main loop.  Step k: scores of half tile k, exponentials of half tile k-1, output product of half
    // tile k-2.  Tile i = half tiles 2i, 2i+1; its K rows and key positions sit in stage i % NST from two tile
    // periods before their first use, its V^T columns from one period later (they are needed a step later and
    // the V^T region of a stage is released a step later).  The first two and the last two steps run the same
    // code on stand-ins: scores of -inf give exponentials of zero, exponentials of zero add nothing, and the
    // scores computed past the last tile are never used.
    const std::integral_constant<int, 0> x0;
    const std::integral_constant<int, 1> x1;
    constexpr int LPT_K = K_INSTR + 1, LPT_V = V_INSTR;
    static_assert(NST == 4, "stage arithmetic");
    volatile int *redo_flags = (volatile int *)(smem + NST * STAGE);   // one word per wavefront
    for (int pass = 0;; ++pass) {                      // one pass, unless an exponent offset had to move late
        redo = false;
        if (pass > 0) first_tiles();
#pragma unroll
        for (int qb = 0; qb < TQ; ++qb) {
            P[0][qb] = P[1][qb] = u32x4{0u, 0u, 0u, 0u};
            // (opaque: zeros rebuilt by moves right in front of the first MFMA that reads them would be read too early)
            if constexpr (SPLIT) asm volatile("" : "+v"(P[0][qb]), "+v"(P[1][qb]));
            L[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) S[0][qb][kb] = S[1][qb][kb] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                O[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
                // (split walk: zeroed here, in the accumulation registers, not inside its conditional loop body)
                if constexpr (SPLIT) asm volatile("" : "+a"(O[qb][db]));
            }
            if constexpr (SPLIT) asm volatile("" : "+a"(L[qb]));
        }
        const std::true_type refill;
        const std::false_type no_refill;
        if constexpr (!SPLIT) {
        phase_barrier<0, false>();                     // everything requested so far is complete and visible
        if (n_tiles > 0) {
#pragma unroll
            for (int f = 0; f < RD; ++f) ring[f] = *(const bf16x8 *)frag_ptr(0, K_BYTES, x0, f);
            int in_flight = 0;                         // loads of this wavefront requested at the previous barrier
            for (int i = 0; i <= n_tiles; ++i) {
                const bool real = i < n_tiles, next_real = i + 1 < n_tiles;
                // past the end: the last tile again (finite scores); in front of the first tile: P is zero
                const int qs = ((real ? i : i - 1) & (NST - 1)) * STAGE;
                const int vs = ((i > 0 ? i - 1 : 0) & (NST - 1)) * STAGE + K_BYTES;
                const int nqs = ((next_real ? i + 1 : i) & (NST - 1)) * STAGE, nvs = (i & (NST - 1)) * STAGE + K_BYTES;
                const bool mask_on = tile_needs_mask(mt0.pmax, mt0.n_rows);
                const bool need0 = step(x0, refill, qs, vs, qs, vs, mask_on);
                between_steps(x0, need0 && real);
                // The barrier between the two steps of a tile: what was requested two barriers ago has landed (the
                // requests of the previous barrier may still be in flight), everyone is past step 2i.  Free from
                // here on: the K region of stage i-1 (last read in step 2i-1), the V^T region of stage i-2 (2i-1).
                __builtin_amdgcn_sched_barrier(0);
                if (in_flight == LPT_K + LPT_V) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LPT_K + LPT_V) : "memory");
                else if (in_flight == LPT_V) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LPT_V) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
                in_flight = 0;
                if (i + 3 < n_tiles) { issue_k(mt3, (i + 3) & (NST - 1)); in_flight += LPT_K; }
                if (i + 2 < n_tiles) { issue_v(mt2, (i + 2) & (NST - 1)); in_flight += LPT_V; }
                const bool need1 = step(x1, refill, qs, vs, nqs, nvs, mask_on);
                between_steps(x1, need1 && real);
                if (real) {
                    if (next_real) mt0 = mt1;
                    mt1 = mt2; mt2 = mt3;
                    if (i + 4 < n_tiles) mt3 = load_meta(i + 4);
                }
            }
        }
        } else {
        // Split walk.  Wavefront group g (0, 1) takes the tiles 2 j + g, j = 0 .. n_g - 1, through two stages of its
        // own (stages 2 g and 2 g + 1); all eight wavefronts load the tiles of both groups.  One barrier in front of
        // every iteration: there K of the tiles j + 1 and V^T of the tiles j are requested (V^T is used an iteration
        // later: the output product trails by a tile), and everything requested at the previous barrier has landed.
        // The operand ring is filled behind the barrier (the second step of an iteration does not read ahead into a
        // tile the barrier has yet to confirm).  Iteration n_g flushes the group's pipeline on a stand-in (its last K
        // tile with every score masked: the query limits are dropped below every position, and fetched again if the
        // pass is repeated); a group with fewer tiles than the other only meets the remaining barriers.
#pragma unroll
        for (int qb = 0; qb < TQ; ++qb) {
            const int rloc = 16 * qb + l16;
            qlim[qb] = p.pos_packed[q_row_start + (rloc < q_n_rows ? rloc : max(q_n_rows - 1, 0))];
        }
        const int n_g0 = (n_tiles + 1) / 2, n_g1 = n_tiles / 2;     // tiles of the two groups; n_g0 >= n_g1
        const int n_mine = rg == 0 ? n_g0 : n_g1, gst = 2 * rg;
        TileMeta &mv0 = mt0, &mv1 = mt1, &mk0 = mt2, &mk1 = mt3;        // tiles j and j + 1 of group 0, of group 1
        for (int j = 0; j <= n_g0; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if (j + 1 < n_g0) issue_k(mk0, (j + 1) & 1);
            if (j + 1 < n_g1) issue_k(mk1, 2 + ((j + 1) & 1));
            if (j < n_g0) issue_v(mv0, j & 1);
            if (j < n_g1) issue_v(mv1, 2 + (j & 1));
            if (n_mine > 0 && j <= n_mine) {
                const bool real = j < n_mine;
                const int qs = (gst + ((real ? j : j - 1) & 1)) * STAGE;
                // in front of the group's first tile the output product (P is zero) reads the K rows: finite numbers
                const int vs = j > 0 ? (gst + ((j - 1) & 1)) * STAGE + K_BYTES : qs;
                if (!real)
#pragma unroll
                    for (int qb = 0; qb < TQ; ++qb) qlim[qb] = -(1 << 30);                 // nothing is visible
#pragma unroll
                for (int f = 0; f < RD; ++f) ring[f] = *(const bf16x8 *)frag_ptr(qs, vs, x0, f);
                // (the flush has every score masked)
                const bool mask_on = !real || (rg == 0 ? tile_needs_mask(mv0.pmax, mv0.n_rows) : tile_needs_mask(mv1.pmax, mv1.n_rows));
                const bool need0 = step(x0, refill, qs, vs, qs, vs, mask_on);
                between_steps(x0, need0 && real);
                const bool need1 = step(x1, no_refill, qs, vs, qs, vs, mask_on);
                between_steps(x1, need1 && real);
            }
            mv0 = mk0; mv1 = mk1;
            if (j + 2 < n_g0) mk0 = load_meta(2 * (j + 2));
            if (j + 2 < n_g1) mk1 = load_meta(2 * (j + 2) + 1);
        }
        }
        mfma_drain();
        // start over together if any wavefront had to move an offset late (the barriers are the workgroup's)
        if (lane == 0) redo_flags[wave] = redo ? 1 : 0;
        phase_barrier<0, true>();
        int any_redo = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) any_redo |= redo_flags[w];
        // (no barrier behind the reads: a flag is written again only at the end of another pass, many barriers away)
        if (!__builtin_amdgcn_readfirstlane(any_redo)) break;
    }

    // ---- split walk: each group keeps half of the head's columns (group 0 the first D/2, group 1 the rest), hands
    // the other half with its offsets and row sums to its partner through LDS (the tile stages are free: everyone is
    // past the last barrier of the pass), merges and writes its half; the offsets are integers, so bringing both to
    // the larger one is exact.  Both groups form the merged row sum from the same operands in the same order.
    if constexpr (SPLIT) {
        constexpr int HB = DB / 2, XW = TQ * HB * 4 + 2 * TQ;      // floats a wavefront hands over per lane
        int o_row[TQ];
#pragma unroll
        for (int qb = 0; qb < TQ; ++qb) {
            const int r = q_row_start + 16 * qb + l16;
            o_row[qb] = p.o_rowmap && row_ok[qb] ? p.o_rowmap[r] : r;
        }
        auto finish_half = [&](auto g_tag) {
            constexpr int G = decltype(g_tag)::value, KEEP = G * HB, GIVE = (1 - G) * HB;
            float *mine = (float *)smem + ((wave % (NWV / 2)) * 2 + G) * (XW * 64) + lane;
            const float *theirs = (const float *)smem + ((wave % (NWV / 2)) * 2 + 1 - G) * (XW * 64) + lane;
#pragma unroll
            for (int qb = 0; qb < TQ; ++qb) {
#pragma unroll
                for (int d = 0; d < HB; ++d)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mine[((qb * HB + d) * 4 + r) * 64] = O[qb][GIVE + d][r];
                mine[(TQ * HB * 4 + qb) * 64] = L[qb][0];
                mine[(TQ * HB * 4 + TQ + qb) * 64] = m_run[qb];
            }
            phase_barrier<-1, true>();
#pragma unroll
            for (int qb = 0; qb < TQ; ++qb) {
                if (!row_ok[qb]) continue;
                const float m1 = theirs[(TQ * HB * 4 + TQ + qb) * 64], l1 = theirs[(TQ * HB * 4 + qb) * 64];
                const float m = fmaxf(m_run[qb], m1);
                const float f0 = m_run[qb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run[qb] - m);
                const float f1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - m);
                const float l_tot = G == 0 ? __builtin_fmaf(l1, f1, L[qb][0] * f0) : __builtin_fmaf(L[qb][0], f0, l1 * f1);
                const float inv = l_tot > 0.f ? __builtin_amdgcn_rcpf(l_tot) : 0.f;
                const float s0 = f0 * inv, s1 = f1 * inv;
                bf16_t *op = p.o + ((int64_t)b * p.N + o_row[qb]) * p.o_ld + (int64_t)h * D + 16 * KEEP + 4 * g4;
#pragma unroll
                for (int d = 0; d < HB; ++d) {
                    f32x4 v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = O[qb][KEEP + d][r] * s0 + theirs[((qb * HB + d) * 4 + r) * 64] * s1;
                    *(bf16x4 *)(op + 16 * d) = bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                }
            }
        };
        if (rg == 0) finish_half(std::integral_constant<int, 0>{});
        else finish_half(std::integral_constant<int, 1>{});
        return;
    }

    // ---- write-out.  O[qb][db][r]: query row 16 qb + l16, column 16 db + 4 g4 + r; every row of L[qb] holds the
    // row sum of query 16 qb + l16.
#pragma unroll
    for (int qb = 0; qb < TQ; ++qb) {
        if (!row_ok[qb]) continue;
        const float l_tot = L[qb][0];
        const int r = q_row_start + wrow0 + 16 * qb + l16;
        const float inv = l_tot > 0.f ? __builtin_amdgcn_rcpf(l_tot) : 0.f;
        bf16_t *op = p.o + ((int64_t)b * p.N + (p.o_rowmap ? p.o_rowmap[r] : r)) * p.o_ld + (int64_t)h * D + 4 * g4;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const f32x4 v = O[qb][db] * inv;
            *(bf16x4 *)(op + 16 * db) = bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
        }
    }
}

template <int D, int TQ, bool MASKED, bool SPLIT = false>
static int32_t launch_fused_cfg(const AttnBf16Params &k, int n_qtiles, hipStream_t s) {
    constexpr int lds = 4 * (KV_TILE * D * 2 + D * 128 + KV_TILE * 4) + 32;   // four stages + the start-over flags
    auto kern = attn_fused_kernel<D, TQ, MASKED, SPLIT>;
    static std::atomic<uint64_t> lds_ready{0};
    CASCADE_HIP_TRY(ensure_dynamic_lds((const void *)kern, lds, lds_ready));
    dim3 grid((unsigned)((int64_t)k.gy * n_qtiles), 1, 1);
    hipLaunchKernelGGL(kern, grid, dim3(1024 / TQ), lds, s, k);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

int32_t launch_attn_fused(const AttnBf16Params &k, int head_dim, int n_qtiles, bool all_visible, bool split, hipStream_t s) {
    if (!k.fused) return CASCADE_EINVAL;
    if (split) {                                       // 32-row query tiles, four heads per workgroup, causal
        if (all_visible || k.hpb != 4) return CASCADE_EINVAL;
        return head_dim == 128 ? launch_fused_cfg<128, 2, true, true>(k, n_qtiles, s) : launch_fused_cfg<64, 2, true, true>(k, n_qtiles, s);
    }
    if (all_visible)
        return head_dim == 128 ? launch_fused_cfg<128, 2, false>(k, n_qtiles, s) : launch_fused_cfg<64, 2, false>(k, n_qtiles, s);
    return head_dim == 128 ? launch_fused_cfg<128, 2, true>(k, n_qtiles, s) : launch_fused_cfg<64, 2, true>(k, n_qtiles, s);
}
