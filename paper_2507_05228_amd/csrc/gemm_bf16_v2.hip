// bf16 shard GEMM, main kernel: Y[rows] = epilogue(X[rows] W^T), fp32 accumulation, K % 64 == 0.
// (The token-as-batch linear layers: q/k/v projection of Algorithm 2, o projection that
// closes Algorithm 4, the MLP step that closes Algorithm 1.  Shards appear only as row maps.)
//
// Shape of the kernel (chosen from measurements on MI355X: 16x16x32 bf16 MFMA reaches ~98 % of the
// chip's matrix peak with two wavefronts per SIMD, ~89 % with one; LDS delivers ~235 B/clk/CU on
// conflict-free 16-byte reads):
//  * 8 wavefronts per workgroup (2 per SIMD, <= 256 registers each) or 4 (one per SIMD, up to 512
//    registers: 128-row wavefront tiles whose accumulators live in the accumulation registers; every
//    memory operation hand-placed between two MFMAs), 16x16x32 MFMA blocks.
//  * K walked in steps of BK (32 or 64).  Tiles go from HBM/L2 straight into LDS with buffer loads
//    that write LDS directly (no register staging, out-of-range rows read as zero), NST stages deep:
//    the loads of steps t+1 .. t+NST-1 are in flight while step t is multiplied.  The wait for "step
//    t has landed" is s_waitcnt vmcnt(loads of the younger steps), issued together with the
//    workgroup barrier as inline assembly: a compiler-generated barrier would wait for vmcnt(0) and
//    drain the pipeline.
//  * LDS rows are BK bf16 without padding; the 16-byte chunk c of tile row r is stored at slot
//    c ^ ((r >> 1) & 7) (128-byte rows) or c ^ ((r >> 2) & 3) (64-byte rows), which makes both the
//    direct-to-LDS writes (1 KiB contiguous per wavefront instruction) and the MFMA operand reads
//    (16 rows x same chunk) bank-conflict free.
//  * Epilogue through LDS.  8 wavefronts: each wavefront transposes 16 accumulator rows at a time so
//    that a lane ends up with 4 consecutive columns (and the 4 columns 64 further on): stores and
//    residual reads are 128-byte runs, and the two halves of a SwiGLU pair live in one lane.
//    4 wavefronts: accumulators are computed transposed (a lane owns 4 consecutive columns already),
//    the bf16 tile of the whole workgroup is laid out in LDS once and stored in 16-byte pieces.
//  * The machine is power-limited under this load (the clock falls from 2.4 to 1.7-2.0 GHz as the
//    matrix pipes fill up), so what counts is energy per flop as much as issue slots: fewer LDS bytes
//    and fewer instructions per MFMA, which is what the 4-wavefront schedule buys.
#include <cstdlib>
#include <type_traits>
#include "common.h"
#include "device_utils.h"
#include "epilogue.h"

#define OOB_OFF 0x80000000u

struct Gemm2Params {
    const bf16_t *X;
    const bf16_t *W[3];
    const bf16_t *bias[3];
    int32_t seg_rows[3], seg_col0[3], seg_tile0[3];
    const bf16_t *Wup;
    const bf16_t *residual;
    bf16_t *Y;
    int32_t M, K;
    int32_t tiles_m, tiles_n;
    int64_t ldx, ldy, ldres;
    const int32_t *xmap, *ymap, *rmap;
    int32_t seq_len, flags;
    uint32_t x_bytes;
    // rotary embedding in the epilogue (ROPE kernels): cos | sin of every packed row's angles, [M][head_dim] fp32;
    // output columns below rope_cols are rotated; rope_lh = log2(head_dim / 2)
    const float *rope_table;
    int32_t rope_cols, rope_lh;
    // split reduction (SPLITK kernels): fp32 partial tiles [tile][accumulator block][thread] and per tile a ticket
    // word and a flag word
    float *sk_partial;
    uint32_t *sk_sync;
};

typedef __attribute__((address_space(3))) void lds_void;


// 16 bytes per lane from a buffer straight into LDS: lane i of the wavefront lands at lds + 16 i.
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t r, unsigned char *lds, uint32_t voff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void *)lds, 16, voff, 0, 0, 0);
}

// Epilogue shared by the shard-GEMM kernels.  acc[i][j][r] holds row 16i + 4(lane/16) + r, column
// 16j + lane%16 of the wavefront's WTM x WTN tile.  The caller guarantees (with a workgroup barrier)
// that every wavefront is done with the tile buffers: smem is reused as staging, one private region
// per wavefront, so inside the epilogue only wavefront-level ordering of LDS traffic is needed.
// SwiGLU pairs (gate column c, up column c + WTN/2) sit in the same lane and register slot, so the
// activation is applied in registers and only WTN/2 columns are staged.
__device__ __forceinline__ float silu_fast(float x) {
    // x * 1/(1 + 2^(-x log2 e)); hardware reciprocal (1 ulp), output is rounded to bf16 anyway
    return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// The residual values a lane adds in gemm_epilogue, all row blocks of its wavefront tile: [row block][row group
// of 4][4-column chunk].
template <int TM, int WTN, bool SWIGLU>
struct ResidualAhead {
    static constexpr int OW = SWIGLU ? WTN / 2 : WTN;
    static constexpr int NCH = (OW + 63) / 64;
    bf16x4 r[TM][4][NCH];
    __device__ __forceinline__ void load(const Gemm2Params &p, int lane, int m0, int wm0, int wn0, int nloc0, int seg,
                                         int seg_rows) {
        const int m4 = (lane & 15) * 4, rsel = lane >> 4;
        const int wcol0 = SWIGLU ? nloc0 + (wn0 / WTN) * OW : nloc0 + wn0;
        const int gcol0 = p.seg_col0[seg];
        const int b0 = m0 / p.seq_len;                     // sequence of the tile's first row (uniform)
        int32_t rows[TM * 4], src[TM * 4];                 // every row's lookup goes out before the first residual load
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int gm = m0 + wm0 + 16 * i + 4 * t + rsel;
                rows[4 * i + t] = gm < p.M ? gm : m0;
            }
        map_rows_near(p.rmap, p.seq_len, rows, b0, src);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int gm = m0 + wm0 + 16 * i + 4 * t + rsel;
                const bf16_t *rrow = p.residual + (int64_t)src[4 * i + t] * p.ldres + gcol0;
#pragma unroll
                for (int cc = 0; cc < NCH; ++cc) {
                    const int c = wcol0 + 64 * cc + m4;
                    r[i][t][cc] = bf16x4{0, 0, 0, 0};
                    if (gm < p.M && c + 4 <= seg_rows && 64 * cc + m4 < OW) r[i][t][cc] = *(const bf16x4 *)(rrow + c);
                }
            }
    }
};

template <int TM, int TN, int WTN, bool SWIGLU>
__device__ __forceinline__ void gemm_epilogue(const Gemm2Params &p, f32x4 (&acc)[TM][TN], unsigned char *smem,
                                              int wave, int lane, int m0, int wm0, int wn0, int nloc0, int seg,
                                              int seg_rows) {
    constexpr bool INREG = SWIGLU && (WTN / 2) % 16 == 0;  // gate and up of a column share lane and slot
    constexpr int OW = SWIGLU ? WTN / 2 : WTN;             // output columns of the wavefront tile
    constexpr int SW = INREG ? OW : WTN;                   // staged columns
    constexpr int TNS = SW / 16;
    constexpr int STG_LD = SW + 4;
    constexpr int NCH = (OW + 63) / 64;                    // 4-column chunks per lane: columns 64 cc + m4
    const int flags = p.flags;
    float *stg = (float *)smem + wave * 16 * STG_LD;
    const int l16 = lane & 15, m4 = l16 * 4, rsel = lane >> 4;
    const int wcol0 = SWIGLU ? nloc0 + (wn0 / WTN) * OW : nloc0 + wn0;   // first output column (in segment)
    const int gcol0 = p.seg_col0[seg];
    const int b0 = m0 / p.seq_len;                         // sequence of the tile's first row (uniform)
    const bf16_t *bias = (flags & CASCADE_EPI_BIAS) ? p.bias[seg] : nullptr;
    f32x4 bias_v[NCH];
#pragma unroll
    for (int cc = 0; cc < NCH; ++cc) {
        const int c = wcol0 + 64 * cc + m4;
        bias_v[cc] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (bias)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (c + x < seg_rows) bias_v[cc][x] = (float)bias[c + x];
    }
    const bool act = flags & (CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH);
    // Residual of every row block requested up front (when the registers allow, if the kernel has not done so
    // ahead of its main loop): one memory latency for the whole epilogue instead of one per row block.
    constexpr bool RES_AHEAD = TM * 4 * NCH <= 32;
    ResidualAhead<RES_AHEAD ? TM : 1, WTN, SWIGLU> res;
    const bool res_ahead = RES_AHEAD && (flags & CASCADE_EPI_RESIDUAL);
    if (res_ahead) res.load(p, lane, m0, wm0, wn0, nloc0, seg, seg_rows);
    // Two copies of the unrolled loops, chosen once: without the (long) GELU code the plain one stays small
    // and contiguous in the instruction cache.
    auto blocks = [&](auto act_tag) {
    constexpr bool ACT = decltype(act_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TNS; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[i][j][r];
                if (INREG) v = silu_fast(v) * acc[i][j + TNS][r];     // SwiGLU launches carry no bias
                stg[(4 * rsel + r) * STG_LD + 16 * j + l16] = v;
            }
        __builtin_amdgcn_wave_barrier();                   // LDS serves one wavefront's accesses in order
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int rl = 4 * t + rsel;
            const int gm = m0 + wm0 + 16 * i + rl;
            if (gm < p.M) {
                bf16_t *yrow = p.Y + map_row_near(p.ymap, p.seq_len, gm, b0) * p.ldy + gcol0;
                const bf16_t *rrow = (flags & CASCADE_EPI_RESIDUAL)
                                         ? p.residual + map_row_near(p.rmap, p.seq_len, gm, b0) * p.ldres + gcol0 : nullptr;
#pragma unroll
                for (int cc = 0; cc < NCH; ++cc) {
                    const int c = wcol0 + 64 * cc + m4;
                    if (c >= seg_rows || 64 * cc + m4 >= OW) continue;
                    f32x4 v = *(const f32x4 *)(stg + rl * STG_LD + 64 * cc + m4);
                    if (!SWIGLU) v += bias_v[cc];
                    if (SWIGLU && !INREG) {
                        const f32x4 up = *(const f32x4 *)(stg + rl * STG_LD + OW + m4);
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = silu_fast(v[x]) * up[x];
                    } else if constexpr (!SWIGLU && ACT) {
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = apply_act_bf16(v[x], flags);
                    }
                    if (c + 4 <= seg_rows) {
                        if (res_ahead) {
                            const bf16x4 rv = res.r[RES_AHEAD ? i : 0][t][cc];
#pragma unroll
                            for (int x = 0; x < 4; ++x) v[x] += (float)rv[x];
                        } else if (rrow) {
                            const bf16x4 rv = *(const bf16x4 *)(rrow + c);
#pragma unroll
                            for (int x = 0; x < 4; ++x) v[x] += (float)rv[x];
                        }
                        bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                        *(bf16x4 *)(yrow + c) = o;
                    } else {
                        for (int x = 0; x < 4 && c + x < seg_rows; ++x)
                            yrow[c + x] = (bf16_t)(v[x] + (rrow ? (float)rrow[c + x] : 0.f));
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    };
    // A tile inside the matrix with no activation to apply takes a copy of the loop without the per-row and
    // per-chunk range checks and with the residual from the registers filled above: a fifth of the instructions.
    // The epilogue of a single-round launch runs once per workgroup, from a cold instruction cache, at about three
    // times the cycles per instruction of warm code, so its length in instructions is what it costs.
    auto blocks_inside = [&](auto res_tag) {
    constexpr bool RES = decltype(res_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TNS; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[i][j][r];
                if (INREG) v = silu_fast(v) * acc[i][j + TNS][r];
                stg[(4 * rsel + r) * STG_LD + 16 * j + l16] = v;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int rl = 4 * t + rsel;
            const int gm = m0 + wm0 + 16 * i + rl;
            bf16_t *yrow = p.Y + map_row_near(p.ymap, p.seq_len, gm, b0) * p.ldy + gcol0 + wcol0 + m4;
#pragma unroll
            for (int cc = 0; cc < NCH; ++cc) {
                f32x4 v = *(const f32x4 *)(stg + rl * STG_LD + 64 * cc + m4);
                if (!SWIGLU) v += bias_v[cc];
                if constexpr (RES) {
                    const bf16x4 rv = res.r[RES_AHEAD ? i : 0][t][cc];
#pragma unroll
                    for (int x = 0; x < 4; ++x) v[x] += (float)rv[x];
                }
                *(bf16x4 *)(yrow + 64 * cc) = bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    };
    constexpr int BN_W = SWIGLU ? OW : WTN;                // output columns per wavefront column
    const bool inside = m0 + wm0 + 16 * TM <= p.M && wcol0 + BN_W <= seg_rows && OW % 64 == 0 && (INREG || !SWIGLU);
    if (inside && !act && RES_AHEAD && (flags & CASCADE_EPI_RESIDUAL)) blocks_inside(std::true_type{});
    else if (inside && !act && !(flags & CASCADE_EPI_RESIDUAL)) blocks_inside(std::false_type{});
    else if (!SWIGLU && act) blocks(std::true_type{});
    else blocks(std::false_type{});
}

// Epilogue for accumulators computed transposed (W block as the first MFMA operand): acc[i][j][r]
// holds row 16i + lane%16, columns 16j + 4(lane/16) + r of the wavefront's tile, so a lane owns four
// consecutive output columns.  Bias, activation, SwiGLU (block j = gate, block j + TN/2 = up: same
// lane, same slot) and the residual are applied in registers, before the one rounding to bf16; the
// result of the whole workgroup tile is laid out row-major in LDS (the tile buffers are free by then)
// and written out in 16-byte pieces that follow each other along the output rows, so every store
// instruction fills whole cache lines.  Row pitch: an odd multiple of 32 bytes, which spreads the 16
// rows of a block write over all banks.
// Accumulator block of the one-wavefront kernels (held in accumulation registers by the tied MFMAs) -> vector
// registers, at the point of use.  Read through plain C++ the compiler copies all blocks across right behind
// the main loop, which a 256-accumulator tile has no registers for.
__device__ __forceinline__ f32x4 acc_load(const f32x4 &c) {
    float x0, x1, x2, x3;
    asm volatile("v_accvgpr_read_b32 %0, %4\n\tv_accvgpr_read_b32 %1, %5\n\tv_accvgpr_read_b32 %2, %6\n\t"
                 "v_accvgpr_read_b32 %3, %7"
                 : "=v"(x0), "=v"(x1), "=v"(x2), "=v"(x3)
                 : "a"(c[0]), "a"(c[1]), "a"(c[2]), "a"(c[3]));
    return f32x4{x0, x1, x2, x3};
}

template <int BN_OUT>
struct EpiTile {
    static constexpr int PITCH = ((BN_OUT * 2 + 31) / 32 | 1) * 32;   // bytes
    static constexpr int bytes(int bm) { return bm * PITCH; }
};
// ROPE: the wavefront tile holds WTN/2 rotation pairs (i, i + head_dim/2 of one head): block j the first
// halves, block j + TN/2 the second halves, same lane and slot, like gate and up of SwiGLU.  The tile's BN
// staged columns are BN/2 first halves followed by their BN/2 partners; pair p of a segment is column
// (p / half) head_dim + p % half and the column `half` further on, so 4 (8) consecutive pairs are 4 (8) consecutive
// columns as long as half is a multiple of 4 (8).  The rotation runs on the fp32 accumulators (one rounding to
// bf16), with cos and sin read from the table the pre-pass norm kernel wrote for every row.
template <int BM, int NTHREADS, int TM, int TN, int WTN, int BN>
__device__ __forceinline__ void gemm_epilogue_tile_rope(const Gemm2Params &p, f32x4 (&acc)[TM][TN], unsigned char *smem,
                                                        int tid, int m0, int wm0, int wn0, int pair0, int seg,
                                                        int seg_rows) {
    static_assert(TN % 2 == 0 && (BN / 2) % 8 == 0, "pairs split the wavefront tile; 16-byte pieces hold 8 pairs");
    constexpr int TNO = TN / 2;
    constexpr int PITCH = EpiTile<BN>::PITCH;
    const int lane = tid & 63, l16 = lane & 15, c4 = (lane >> 4) * 4;
    const int wp0 = (wn0 / WTN) * (WTN / 2);               // wavefront's first pair inside the tile
    const int lh = p.rope_lh, half = 1 << lh, n_pairs = seg_rows >> 1;
    const int gcol0 = p.seg_col0[seg];
    const int b0 = m0 / p.seq_len;                         // sequence of the tile's first row (uniform)
    const bf16_t *bias = (p.flags & CASCADE_EPI_BIAS) ? p.bias[seg] : nullptr;
    f32x4 bias_a[TNO], bias_b[TNO];                        // of this lane's pairs, once
#pragma unroll
    for (int j = 0; j < TNO; ++j) {
        const int pp = pair0 + wp0 + 16 * j + c4;
        const int col1 = ((pp >> lh) << (lh + 1)) + (pp & (half - 1));
        bias_a[j] = bias_b[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (bias && pp < n_pairs) {
            const bf16x4 a4 = *(const bf16x4 *)(bias + col1), b4 = *(const bf16x4 *)(bias + col1 + half);
            bias_a[j] = f32x4{(float)a4[0], (float)a4[1], (float)a4[2], (float)a4[3]};
            bias_b[j] = f32x4{(float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]};
        }
    }
    // A tile inside the matrix, without bias, whose columns are all rotated (q, k) or all passed through (v) takes a
    // copy of the loop without the per-pair checks, with the cos | sin values requested three row blocks ahead
    // (2 x 16 bytes per pair block and row from the table in L2: one latency instead of one per row block).  The
    // code runs once per workgroup, from a cold instruction cache: its length in instructions is what it costs.
    auto stage1_inside = [&](auto rot_tag) {
        constexpr bool ROT = decltype(rot_tag)::value;
        constexpr int AH = ROT ? (TNO > 4 ? 2 : 3) : 1;       // 8 registers per pair block and row block in flight
        f32x4 cs[AH][ROT ? TNO : 1], sn[AH][ROT ? TNO : 1];
        auto request = [&](int i) {
            if constexpr (ROT) {
                const float *trow = p.rope_table + (int64_t)(m0 + wm0 + 16 * i + l16) * (2 * half);
#pragma unroll
                for (int j = 0; j < TNO; ++j) {
                    const int ph = (pair0 + wp0 + 16 * j + c4) & (half - 1);
                    cs[i % AH][j] = *(const f32x4 *)(trow + ph);
                    sn[i % AH][j] = *(const f32x4 *)(trow + half + ph);
                }
            }
        };
#pragma unroll
        for (int i = 0; i < AH - 1 && i < TM; ++i) request(i);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm0 + 16 * i + l16;
            if (i + AH - 1 < TM) request(i + AH - 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TNO; ++j) {
                const int tp = wp0 + 16 * j + c4;
                f32x4 a = acc_load(acc[i][j]), b = acc_load(acc[i][j + TNO]);
                if constexpr (ROT) {
                    const f32x4 c = cs[i % AH][j], sv = sn[i % AH][j];
                    const f32x4 ra = a * c - b * sv, rb = b * c + a * sv;
                    a = ra; b = rb;
                }
                *(bf16x4 *)(smem + row * PITCH + tp * 2) = bf16x4{(bf16_t)a[0], (bf16_t)a[1], (bf16_t)a[2], (bf16_t)a[3]};
                *(bf16x4 *)(smem + row * PITCH + (BN / 2 + tp) * 2) = bf16x4{(bf16_t)b[0], (bf16_t)b[1], (bf16_t)b[2], (bf16_t)b[3]};
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // columns of the tile: whole heads from the head of its first pair to the head of its last
    const int col_lo = gcol0 + ((pair0 >> lh) << (lh + 1)), col_hi = gcol0 + ((((pair0 + BN / 2 - 1) >> lh) + 1) << (lh + 1));
    const bool tile_inside = m0 + BM <= p.M && pair0 + BN / 2 <= n_pairs && !bias;
    if (tile_inside && col_hi <= p.rope_cols) stage1_inside(std::true_type{});
    else if (tile_inside && col_lo >= p.rope_cols) stage1_inside(std::false_type{});
    else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = wm0 + 16 * i + l16, gm = m0 + row;
        const float *trow = p.rope_table + (int64_t)(gm < p.M ? gm : 0) * (2 * half);
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
            const int tp = wp0 + 16 * j + c4;              // pair inside the tile; 4 consecutive pairs, one head
            const int pp = pair0 + tp, ph = pp & (half - 1);
            const int col1 = ((pp >> lh) << (lh + 1)) + ph;
            const bool inside = pp < n_pairs;
            f32x4 a = acc_load(acc[i][j]) + bias_a[j], b = acc_load(acc[i][j + TNO]) + bias_b[j];
            if (inside && gcol0 + col1 < p.rope_cols) {
                const f32x4 cs = *(const f32x4 *)(trow + ph), sn = *(const f32x4 *)(trow + half + ph);
                const f32x4 ra = a * cs - b * sn, rb = b * cs + a * sn;
                a = ra; b = rb;
            }
            *(bf16x4 *)(smem + row * PITCH + tp * 2) = bf16x4{(bf16_t)a[0], (bf16_t)a[1], (bf16_t)a[2], (bf16_t)a[3]};
            *(bf16x4 *)(smem + row * PITCH + (BN / 2 + tp) * 2) = bf16x4{(bf16_t)b[0], (bf16_t)b[1], (bf16_t)b[2], (bf16_t)b[3]};
        }
    }
    }
    __syncthreads();
    constexpr int CPRO = BN / 8;                           // 16-byte pieces per tile row
    const bool wide = ((p.ldy | gcol0) % 8 == 0) && ((uintptr_t)p.Y % 16 == 0);
    // A thread keeps its piece of the row (CPRO pieces per row: its column offset is computed once) and walks down
    // the rows RPP at a time; the LDS reads (and row-map lookups) of a group of pieces are in flight before the
    // group's first store.
    constexpr int RPP = NTHREADS / CPRO, NPASS = (BM + RPP - 1) / RPP, GRP = 8;
    static_assert(CPRO <= NTHREADS, "a row of pieces per pass at least");
    const int trow = tid / CPRO, piece = tid - trow * CPRO;
    const int hs = piece >= CPRO / 2;                      // second halves
    const int pp = pair0 + (piece - hs * (CPRO / 2)) * 8;
    const int c = ((pp >> lh) << (lh + 1)) + (pp & (half - 1)) + (hs << lh);
    const bool t_ok = trow < RPP && pp < n_pairs;          // n_pairs is a multiple of half, half of 8
    const bool rows_inside = m0 + BM <= p.M;
    const unsigned char *src = smem + trow * PITCH + piece * 16;
#pragma unroll
    for (int g0 = 0; g0 < NPASS; g0 += GRP) {
        bf16x8 v[GRP];
        bf16_t *y[GRP];
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            const int row = (g0 + g) * RPP + trow, gm = m0 + row;
            y[g] = nullptr;
            if (g0 + g >= NPASS || !t_ok || row >= BM || (!rows_inside && gm >= p.M)) continue;
            v[g] = *(const bf16x8 *)(src + (g0 + g) * RPP * PITCH);
            y[g] = p.Y + map_row_near(p.ymap, p.seq_len, gm, b0) * p.ldy + gcol0 + c;
        }
#pragma unroll
        for (int g = 0; g < GRP; ++g) {
            if (g0 + g >= NPASS || !y[g]) continue;
            if (wide) {
                *(bf16x8 *)y[g] = v[g];
            } else {
                *(bf16x4 *)y[g] = bf16x4{v[g][0], v[g][1], v[g][2], v[g][3]};
                *(bf16x4 *)(y[g] + 4) = bf16x4{v[g][4], v[g][5], v[g][6], v[g][7]};
            }
        }
    }
}

// PARTNER (split reduction, the workgroup that finishes the tile): the other workgroup's accumulators, stored at
// `part` as they lay in its registers, are added to this one's in stage 1; they are valid once the word at
// `flag` reads `use`, which is waited for as late as possible, after the row lookups of stage 2 are on their way.
template <int BM, int NTHREADS, int TM, int TN, int WTN, bool SWIGLU, int BN_OUT, bool ACT_OK, bool PARTNER = false>
__device__ __forceinline__ void gemm_epilogue_tile(const Gemm2Params &p, f32x4 (&acc)[TM][TN], unsigned char *smem,
                                                   int tid, int m0, int wm0, int wn0, int nloc0, int seg,
                                                   int seg_rows, const f32x4 *part = nullptr, uint32_t *flag = nullptr,
                                                   uint32_t use = 0) {
    static_assert(!SWIGLU || TN % 2 == 0, "gate and up blocks pair up inside the wavefront tile");
    static_assert(!PARTNER || !SWIGLU, "the split reduction runs plain GEMMs");
    constexpr int TNO = SWIGLU ? TN / 2 : TN;              // output blocks of the wavefront tile
    constexpr int OW = SWIGLU ? WTN / 2 : WTN;
    constexpr int PITCH = EpiTile<BN_OUT>::PITCH;
    const int flags = p.flags;
    const int lane = tid & 63, l16 = lane & 15, c4 = (lane >> 4) * 4;
    const int wc0 = (wn0 / WTN) * OW;                      // wavefront's first output column inside the tile
    const bf16_t *bias = (!SWIGLU && (flags & CASCADE_EPI_BIAS)) ? p.bias[seg] : nullptr;
    const bool act = ACT_OK && (flags & (CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH));
    const int gcol0 = p.seg_col0[seg];
    const int b0 = m0 / p.seq_len;                         // sequence of the tile's first row (uniform)
    const bool has_res = flags & CASCADE_EPI_RESIDUAL;
    // 16-byte stores need the rows to start on 16-byte boundaries; otherwise two 8-byte halves
    const bool wide = ((p.ldy | gcol0) % 8 == 0) && ((uintptr_t)p.Y % 16 == 0);
    // One wavefront per SIMD: the epilogue is as long as its instruction count, nothing overlaps it.  A tile that
    // lies inside the matrix (all but the last row and column of tiles) takes copies of the two loops without any
    // of the per-element range checks, chosen once per tile; so does the choice between residual and none.
    const bool interior = m0 + BM <= p.M && nloc0 + BN_OUT <= seg_rows && wide;
    // Stage 1, accumulators -> bf16 tile in LDS.  GENERAL: bias and activation code present.  INTERIOR: no range
    // checks.  RES: 0 no residual, 1 residual, 2 decided at run time.
    // The residual of row block i + RES_AHEAD - 1 is requested before row block i is worked on (RES_AHEAD register
    // sets of 2 TNO registers: the whole tile's residual costs about one memory latency, not one per row block;
    // with two sets the second workgroup of a split reduction spent 46 k cycles in this epilogue, half of them
    // waiting), and the compiler may not move anything across the row-block boundaries: left alone it hoists the
    // loads and the accumulator reads of all blocks to the top, which the 256-accumulator tile has no registers for.
    auto to_lds = [&](auto general_tag, auto interior_tag, auto res_tag) {
    constexpr bool GENERAL = decltype(general_tag)::value, INTERIOR = decltype(interior_tag)::value;
    constexpr int RES = decltype(res_tag)::value;
    const bool res = RES == 2 ? has_res : RES == 1;
    constexpr int RES_AHEAD = TM < 5 ? TM : 5;
    bf16x4 rv[RES_AHEAD][TNO];
    auto load_res = [&](int i, int buf) {
        const int gm = m0 + wm0 + 16 * i + l16;
        const bf16_t *rrow = p.residual + map_row_near(p.rmap, p.seq_len, INTERIOR || gm < p.M ? gm : 0, b0) * p.ldres + gcol0 + nloc0;
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
            const int tc = wc0 + 16 * j + c4;
            if (INTERIOR) rv[buf][j] = *(const bf16x4 *)(rrow + tc);
            else {
                rv[buf][j] = bf16x4{0, 0, 0, 0};
                if (gm < p.M && nloc0 + tc < seg_rows) rv[buf][j] = *(const bf16x4 *)(rrow + tc);
            }
        }
    };
    // the bias of this lane's columns, once (it does not depend on the row block)
    f32x4 bias_v[GENERAL ? TNO : 1];
    if constexpr (GENERAL) {
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
            const int tc = wc0 + 16 * j + c4;
            bias_v[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (bias && nloc0 + tc < seg_rows) {
                const bf16x4 b4 = *(const bf16x4 *)(bias + nloc0 + tc);
                bias_v[j] = f32x4{(float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]};
            }
        }
    }
    // the partner's accumulators, three row blocks ahead like the residual
    constexpr int P_AHEAD = PARTNER ? (TM < 3 ? TM : 3) : 1;
    f32x4 pvv[P_AHEAD][PARTNER ? TNO : 1];
    auto load_part = [&](int i) {
        if constexpr (PARTNER)
#pragma unroll
            for (int j = 0; j < TNO; ++j) pvv[i % P_AHEAD][j] = __builtin_nontemporal_load(part + (i * TN + j) * NTHREADS);
    };
    if constexpr (PARTNER)
#pragma unroll
        for (int i = 0; i < P_AHEAD - 1 && i < TM; ++i) load_part(i);
    if (res)
#pragma unroll
        for (int i = 0; i < RES_AHEAD - 1 && i < TM; ++i) load_res(i, i % RES_AHEAD);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = wm0 + 16 * i + l16;
        if (PARTNER && i + P_AHEAD - 1 < TM) load_part(i + P_AHEAD - 1);
        if (res && i + RES_AHEAD - 1 < TM) load_res(i + RES_AHEAD - 1, (i + RES_AHEAD - 1) % RES_AHEAD);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
            const int tc = wc0 + 16 * j + c4;              // column inside the tile
            f32x4 v = acc_load(acc[i][j]);
            if constexpr (PARTNER) v += pvv[i % P_AHEAD][j];
            if constexpr (SWIGLU) {
                const f32x4 up = acc_load(acc[i][j + TNO]);
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = silu_fast(v[x]) * up[x];
            } else if constexpr (GENERAL) {
                v += bias_v[j];
                if constexpr (ACT_OK)
                    if (act)
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = apply_act_bf16(v[x], flags);
            }
            if (res) {                                     // added before the one rounding to bf16
                const bf16x4 r4 = rv[i % RES_AHEAD][j];
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] += (float)r4[x];
            }
            const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
            *(bf16x4 *)(smem + row * PITCH + tc * 2) = o;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    };
    // Stage 2's rows, looked up now where the output is scattered through a row map: the lookups are in flight
    // while stage 1 runs instead of in front of every group of stores.
    constexpr int CPRO = BN_OUT / 8;                       // 16-byte pieces per tile row
    static_assert(BN_OUT % 8 == 0 && CPRO <= NTHREADS, "whole pieces");
    constexpr int RPP = NTHREADS / CPRO, NPASS = (BM + RPP - 1) / RPP, GRP = 8;
    const int trow = tid / CPRO, piece = tid - trow * CPRO;
    int yrow[NPASS];                                       // output row of pass g (negative: nothing to store)
#pragma unroll
    for (int g = 0; g < NPASS; ++g) {
        const int row = g * RPP + trow, gm = m0 + row;
        yrow[g] = (trow < RPP && row < BM && gm < p.M) ? (int)map_row_near(p.ymap, p.seq_len, gm, b0) : -1;
    }
    if constexpr (PARTNER) {
        // One wavefront polls and acquires (an acquire invalidates a whole L2); the workgroup barrier orders the
        // other wavefronts' loads behind it.  The partner holds its ticket already: it is running and waits for
        // nothing, so the wait ends (the spin count only guards against a partner that died).
        if (tid == 0) {
            int spins = 0;
            while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != use && ++spins < (1 << 22))
                __builtin_amdgcn_s_sleep(8);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
    }
    const std::integral_constant<int, 0> res_no;
    const std::integral_constant<int, 1> res_yes;
    const std::integral_constant<int, 2> res_rt;
    if (!SWIGLU && (bias || act)) to_lds(std::true_type{}, std::false_type{}, res_rt);
    else if (!interior) to_lds(std::false_type{}, std::false_type{}, res_rt);
    else if (has_res) to_lds(std::false_type{}, std::true_type{}, res_yes);
    else to_lds(std::false_type{}, std::true_type{}, res_no);
    __syncthreads();
    // Stage 2, LDS tile -> global in 16-byte pieces.  A thread keeps its piece of the row (CPRO pieces per row) and
    // walks down the rows RPP at a time, so the only per-piece work is an LDS read, a row-map lookup where the
    // output is scattered, one address addition and the store; the reads (and lookups) of a group of pieces are
    // in flight before the group's first store.
    const int c = nloc0 + piece * 8;
    const unsigned char *src = smem + trow * PITCH + piece * 16;
    auto store_tile = [&](auto interior_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
        const bool t_ok = INTERIOR || c < seg_rows;
        const bool whole = INTERIOR || c + 8 <= seg_rows;  // else the segment ends inside this piece
#pragma unroll
        for (int g0 = 0; g0 < NPASS; g0 += GRP) {
            bf16x8 v[GRP];
            bf16_t *y[GRP];
#pragma unroll
            for (int g = 0; g < GRP; ++g) {
                y[g] = nullptr;
                if (g0 + g >= NPASS) continue;
                if (!t_ok || yrow[g0 + g < NPASS ? g0 + g : 0] < 0) continue;
                v[g] = *(const bf16x8 *)(src + (g0 + g) * RPP * PITCH);
                y[g] = p.Y + (int64_t)yrow[g0 + g < NPASS ? g0 + g : 0] * p.ldy + gcol0 + c;
            }
#pragma unroll
            for (int g = 0; g < GRP; ++g) {
                if (g0 + g >= NPASS || !y[g]) continue;
                if (INTERIOR || (whole && wide)) {
                    *(bf16x8 *)y[g] = v[g];
                } else if (whole) {
                    *(bf16x4 *)y[g] = bf16x4{v[g][0], v[g][1], v[g][2], v[g][3]};
                    *(bf16x4 *)(y[g] + 4) = bf16x4{v[g][4], v[g][5], v[g][6], v[g][7]};
                } else {
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (c + x < seg_rows) y[g][x] = v[g][x];
                }
            }
        }
    };
    if (interior) store_tile(std::true_type{});
    else store_tile(std::false_type{});
}

// Tile number -> tile coordinates.  Row tiles run fastest inside groups of 8 rows of tiles, column tiles next, groups
// last: the 32 consecutive tiles an XCD works on at a time are then 8 row tiles x 4 column tiles (every activation
// tile shared by 4 workgroups through the XCD's L2, every weight tile by 8), however many rows of tiles the
// launch has; with up to 8 rows of tiles this is the plain row-fastest order.
__device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int &tile_m, int &tile_n) {
    constexpr int GM = 8;                                  // 16 and 4 measured 1 % slower at 32 rows of tiles
    const int width = GM * tiles_n, group = tile / width, first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM), in_group = tile - group * width;
    tile_m = first_m + in_group % gsz;
    tile_n = in_group / gsz;
}

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    // all but the N youngest vector-memory operations of this wavefront are complete and its LDS reads
    // have returned, then barrier
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// MFMA with the accumulator tied to the destination and held in the accumulation registers.  Used by
// the one-wavefront-per-SIMD schedule, where the 224-256 accumulator registers of a 128-row wavefront
// tile only fit there; written as assembly so that source and destination stay the same registers and
// so that the hand-placed operand reads and tile loads keep their place between the MFMAs (the
// compiler does not move memory operations across these statements).
__device__ __forceinline__ void mfma_tied(f32x4 &c, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
// The compiler does not see those MFMAs: before anything else reads the accumulators, let the last
// ones leave the matrix pipeline.
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

// The lane number from the execution mask, as assembly: the compiler can neither tell that it is threadIdx.x % 64
// nor merge two of these, so nothing is kept in a register between them.
__device__ __forceinline__ int lane_id_again() {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// Reduction split over two workgroups per tile (a launch whose tiles would fill half of the CUs).  Each computes
// one half of K into its accumulators.  Then it takes a ticket from the tile's counter: the holder of the even
// ticket (the first to finish) writes its accumulators to the tile's slot of the scratch as they lie in its
// registers, publishes them by setting the tile's flag to the use count of the slot (returned in `use`), and is
// done; the holder of the odd ticket returns true: it runs the epilogue, which waits for that flag and adds the
// stored accumulators to its own.  The workgroup that is waited for took its ticket earlier, so it is running, has its main loop
// behind it and waits for nothing itself: the wait ends whatever the order in which workgroups are placed on the
// CUs (the spin count only guards against a partner that died).  Ticket and flag count up over the launches that
// share the words (which run one after the other), so nothing has to be reset between them.
template <int TM, int TN, int NTHREADS>
__device__ __forceinline__ bool splitk_combine(const Gemm2Params &p, f32x4 (&acc)[TM][TN], int tile, int tid,
                                               unsigned char *smem, uint32_t &use_out) {
    uint32_t *sync = p.sk_sync + 2 * tile;
    f32x4 *part = (f32x4 *)p.sk_partial + (size_t)tile * (TM * TN * NTHREADS) + tid;
    volatile uint32_t *sh = (volatile uint32_t *)smem;
    if (tid == 0) sh[0] = __hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t ticket = sh[0];
    const uint32_t use = (ticket >> 1) + 1;
    use_out = use;
    // Cache maintenance across the XCDs' L2s is expensive (a release writes back, an acquire invalidates a whole
    // L2), so exactly one wavefront of each workgroup does it: the workgroup barrier orders the other wavefronts'
    // stores before thread 0's release and their loads after thread 0's acquire.
    if ((ticket & 1u) == 0u) {
        // stored straight from the accumulation registers (a vector-memory instruction takes them as data): this
        // runs once, on the path the other workgroup waits for, and 256 register moves less is a third of it
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                asm volatile("global_store_dwordx4 %0, %1, off" ::"v"(part + (i * TN + j) * NTHREADS), "a"(acc[i][j]) : "memory");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the compiler does not count those stores
        __syncthreads();
        if (tid == 0) __hip_atomic_store(&sync[1], use, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    return true;
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool SWIGLU, bool ROPE = false, bool SPLITK = false>
__global__ __launch_bounds__(WM *WN * 64) void gemm2_kernel(Gemm2Params p) {
    static_assert(!ROPE || (!SWIGLU && WM * WN == 4), "rotary epilogue: plain GEMM, one wavefront per SIMD");
    static_assert(!SPLITK || (!SWIGLU && !ROPE && WM * WN == 4), "split reduction: plain GEMM, one wavefront per SIMD");
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 16, TN = WTN / 16;
    constexpr bool SOLO = NW == 4;                                 // one wavefront per SIMD, up to 512 registers
    constexpr int ROWB = BK * 2;                                   // bytes per tile row in LDS
    constexpr int RPI = 1024 / ROWB;                               // tile rows per direct-to-LDS instruction
    constexpr int CPR = ROWB / 16;                                 // 16-byte chunks per row
    constexpr int BNP = (BN + RPI * NW - 1) / (RPI * NW) * (RPI * NW);   // B rows held in LDS (BN rounded up)
    constexpr int A_INSTR = BM / RPI / NW, B_INSTR = BNP / RPI / NW;     // direct-to-LDS instructions per wavefront
    constexpr int LPT = A_INSTR + B_INSTR;                         // loads per tile per wavefront
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BNP) * ROWB;
    constexpr int STG_LD = WTN + 4;                                // widest epilogue staging row (floats)
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(NST >= 2 && NST <= 4 && (NST - 2) * LPT < 64, "pipeline depth");
    static_assert(BM % (RPI * NW) == 0, "tile rows must split over the wavefronts");
    static_assert(WTN % 16 == 0 && (SOLO || WTN <= 128) && BN % RPI == 0, "wavefront tile: whole MFMA blocks, at most 128 columns");
    static_assert(!SWIGLU || ((WTN / 2) % RPI == 0 && (WTN / 2) % 4 == 0),
                  "a load instruction / a store chunk must not straddle gate and up rows");
    static_assert(SOLO || NW * 16 * STG_LD * 4 <= NST * STAGE_BYTES, "epilogue staging must fit in the tile buffers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

    // workgroup -> tile: a contiguous run of the tile list per XCD (see tile_coords for the order of the list)
    // One wavefront per SIMD: the workgroup is persistent.  The launch has one workgroup per CU (a multiple of 8)
    // and workgroup w takes the tiles that workgroups w, w + gridDim.x, ... of a launch with one workgroup per
    // tile would take: nothing waits for a workgroup's last stores to be acknowledged, for its registers and LDS
    // to be handed on, or for a new workgroup to set itself up; the stores of a tile drain while the first
    // tile loads of the next are in flight.
    constexpr bool PERSISTENT = SOLO && !SPLITK;
    const int total = p.tiles_m * p.tiles_n;
    for (int pid = blockIdx.x;; pid += gridDim.x) {
    int tile, khalf = 0;
    if constexpr (SPLITK) {                                        // total % 8 == 0; the two halves of a tile are
        const int xcd = pid & 7, idx = pid >> 3;                   // neighbours in the dispatch order of one XCD
        tile = xcd * (total >> 3) + (idx >> 1);
        khalf = idx & 1;
    } else {
        const int xcd = pid & 7, idx = pid >> 3;
        const int base = total >> 3, rem = total & 7;
        tile = xcd * base + min(xcd, rem) + idx;
    }
    int tile_m, tile_n;
    tile_coords(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int seg = tile_n >= p.seg_tile0[2] ? 2 : tile_n >= p.seg_tile0[1] ? 1 : 0;
    const int m0 = tile_m * BM;
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    const int nloc0 = (tile_n - p.seg_tile0[seg]) * BN_OUT;
    const int seg_rows = p.seg_rows[seg];
    const int K = p.K;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.X), 0, p.x_bytes, 0x00020000);
    const uint32_t w_bytes = (uint32_t)((int64_t)seg_rows * K * 2);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.W[seg]), 0, w_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ru =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(SWIGLU ? p.Wup : p.W[seg]), 0, w_bytes, 0x00020000);

    // ---- per-lane global offsets of the direct-to-LDS loads.  Instruction i of this wavefront fills
    // tile rows wave*(rows/NW) + RPI*i .. : lane -> row lane/CPR, LDS slot lane%CPR, which must hold the
    // logical chunk slot ^ swizzle(row).
    auto swz = [](int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    uint32_t a_off[A_INSTR], b_off[B_INSTR];
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
        const int row = wave * (BM / NW) + RPI * i + lane / CPR;
        const int c = (lane % CPR) ^ swz(row);
        const int gm = m0 + row;
        a_off[i] = gm < p.M ? (uint32_t)(map_row_near(p.xmap, p.seq_len, gm, m0 / p.seq_len) * p.ldx * 2) + c * 16 : OOB_OFF;
    }
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
        const int row = wave * (BNP / NW) + RPI * i + lane / CPR;
        const int c = (lane % CPR) ^ swz(row);
        int col;
        if (SWIGLU) col = nloc0 + (row / WTN) * (WTN / 2) + (row % (WTN / 2));
        else if (ROPE) {                                           // tile row -> rotation pair and half of it
            const int rr = row % WTN, hs = rr / (WTN / 2);
            const int pp = (nloc0 >> 1) + (row / WTN) * (WTN / 2) + rr % (WTN / 2);
            const int lh = p.rope_lh;
            col = pp < (seg_rows >> 1) ? ((pp >> lh) << (lh + 1)) + (pp & ((1 << lh) - 1)) + (hs << lh) : seg_rows;
        } else col = nloc0 + row;
        b_off[i] = (row < BN && col < seg_rows) ? (uint32_t)((int64_t)col * K * 2) + c * 16 : OOB_OFF;
    }

    // LDS layout.  8 wavefronts: NST stages of [A tile | B tile].  One wavefront per SIMD: three A stages
    // followed by two B stages (the A part of a refill is issued half a tile earlier than the B part, so the
    // vector-memory instructions are spread over both k-steps; that needs the third A stage).
    constexpr int B_BYTES = BNP * ROWB;
    constexpr int NSTA = 3, NSTB = 2;
    auto a_stage = [&](int kt) { return SOLO ? smem + (kt % NSTA) * A_BYTES : smem + (kt % NST) * STAGE_BYTES; };
    auto b_stage = [&](int kt) {
        return SOLO ? smem + NSTA * A_BYTES + (kt % NSTB) * B_BYTES : smem + (kt % NST) * STAGE_BYTES + A_BYTES;
    };
    const int KT = SPLITK ? K / BK / 2 : K / BK;                   // k-tiles of this workgroup
    if constexpr (SPLITK) {                                        // the second half starts KT k-tiles in (offsets of
        const uint32_t koff = (uint32_t)(khalf * KT) * ROWB;       // rows outside stay outside: K bytes < 2^31)
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) a_off[i] += koff;
#pragma unroll
        for (int i = 0; i < B_INSTR; ++i) b_off[i] += koff;
    }
    auto issue_load = [&](int kt, int stage, int x) {              // instruction x of LPT (x known after unrolling)
        const uint32_t kb = (uint32_t)kt * ROWB;
        (void)stage;                                               // = kt % NST for the 8-wavefront layout
        if (x < A_INSTR) {
            unsigned char *sa = a_stage(kt) + wave * (BM / NW) * ROWB;
            load16_to_lds(rx, sa + x * 1024, a_off[x] + kb);
        } else {
            const int i = x - A_INSTR;
            unsigned char *sb = b_stage(kt) + wave * (BNP / NW) * ROWB;
            const int row0 = wave * (BNP / NW) + RPI * i;                   // wavefront-uniform
            const bool up = SWIGLU && ((row0 % WTN) >= WTN / 2);
            if (up) load16_to_lds(ru, sb + i * 1024, b_off[i] + kb);
            else load16_to_lds(rw, sb + i * 1024, b_off[i] + kb);
        }
    };
    auto issue_loads = [&](int kt, int stage) {
#pragma unroll
        for (int x = 0; x < LPT; ++x) issue_load(kt, stage, x);
    };

    f32x4 acc[TM][TN];

    // operand fetch: lane -> tile row lane%16 of a 16-row block, chunk 4 ks + lane/16, swizzled
    const int frow = lane & 15, fch = lane >> 4, fsw = swz(lane & 15);
    const int a_lane = (wm0 + frow) * ROWB, b_lane = A_BYTES + (wn0 + frow) * ROWB;
    constexpr int KS = BK / 32;
    static_assert(KS == 2, "the operand pipeline below alternates two register sets over the two k-steps of a tile");
    constexpr int NSETS = SOLO || 4 * TM * TN + 8 * (TM + TN) <= 216 ? 2 : 1;
    bf16x8 af[NSETS][TM], bfr[NSETS][TN];
    auto fetch_into = [&](int kt, auto set_tag, auto ks_tag) {   // operands of k-step ks of tile kt -> register set
        constexpr int set = decltype(set_tag)::value, ks = decltype(ks_tag)::value;
        const unsigned char *st = smem + (kt % NST) * STAGE_BYTES;
        const int coff = ((4 * ks + fch) ^ fsw) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[set][i] = *(const bf16x8 *)(st + a_lane + i * 16 * ROWB + coff);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[set][j] = *(const bf16x8 *)(st + b_lane + j * 16 * ROWB + coff);
    };
    auto mfmas = [&](auto ks_tag) {
        constexpr int ks = decltype(ks_tag)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
    };
    // Tile kt has landed once at most the loads of the younger tiles in flight are outstanding; the
    // wavefront's own LDS reads have returned (they were of the tile whose stage is refilled next);
    // after the barrier every wavefront is done reading tile kt-1.
    auto tile_ready = [&](int kt) {
        const int younger = min(NST - 2, KT - 1 - kt);
        if (younger >= 2) wait_loads_and_barrier<2 * LPT>();
        else if (younger == 1) wait_loads_and_barrier<LPT>();
        else wait_loads_and_barrier<0>();
        if (kt + NST - 1 < KT) issue_loads(kt + NST - 1, (kt + NST - 1) % NST);
    };
    const std::integral_constant<int, 0> k0;
    const std::integral_constant<int, 1> k1;
#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < KT) issue_loads(s, s);
    // One wavefront per SIMD: its A and B stages hold two tiles apart from the one being multiplied, so the second
    // k-tile is requested right behind the first (requested only once the first had landed, its latency sat in
    // front of the first barrier of every output tile).
    if constexpr (SOLO)
        if (1 < KT) issue_loads(1, 1);
    // (the accumulators are cleared while the first tile loads are in flight: up to 256 register writes)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    __builtin_amdgcn_sched_barrier(0);
    // Software pipeline over k-steps: the LDS reads of a k-step are in flight while the MFMAs of the
    // previous k-step run, also across the tile boundary (the second k-step of tile kt is multiplied
    // after the barrier that opens tile kt+1, from registers).  It needs two operand register sets;
    // the widest tile (256 columns: 128 accumulator + 96 operand registers) would spill with them and
    // keeps one k-step's reads directly ahead of its own MFMAs instead.
    constexpr bool PIPE = 4 * TM * TN + 8 * (TM + TN) <= 216;
    if constexpr (SOLO) {                                          // tile 0 has landed; tile 1 may be on its way
        if (1 < KT) wait_loads_and_barrier<LPT>();
        else wait_loads_and_barrier<0>();
    } else tile_ready(0);
    if constexpr (SOLO) {
        // One wavefront per SIMD: nothing else covers this wavefront's waits, so every memory operation
        // is placed between two MFMAs of the k-step that runs meanwhile.  Tile kt, first k-step: its
        // MFMAs with the operand reads of the second k-step (all issued in the first half, so that they
        // have returned at the barrier) and the A loads of tile kt+2 (into the A stage tile kt-1 left)
        // between them.  Barrier (tile kt+1 landed: everything but those A loads; everyone is done reading
        // tile kt).  Second k-step: its MFMAs with the B loads of tile kt+2 (into the B stage tile kt just
        // left) and the operand reads of tile kt+1's first k-step between them.
        static_assert(NST == 2, "the prologue requests tiles 0 and 1");
        constexpr int NR = TM + TN;
        static_assert(2 * NR <= TM * TN && 2 * A_INSTR <= TM * TN && 2 * B_INSTR <= TM * TN,
                      "one read and one load per two MFMAs");
        auto fetch_one = [&](int kt, auto ks_tag, int r) {     // read r of a k-step: A block 0, the B blocks, the other A blocks
            constexpr int ks = decltype(ks_tag)::value;
            const unsigned char *sa = a_stage(kt) + a_lane, *sb = b_stage(kt) + (b_lane - A_BYTES);
            const int coff = ((4 * ks + fch) ^ fsw) * 16;
            if (r == 0) af[ks][0] = *(const bf16x8 *)(sa + coff);
            else if (r <= TN) bfr[ks][r - 1] = *(const bf16x8 *)(sb + (r - 1) * 16 * ROWB + coff);
            else af[ks][r - TN] = *(const bf16x8 *)(sa + (r - TN) * 16 * ROWB + coff);
        };
        auto phase = [&](auto ks_tag, auto &&between) {        // the MFMAs of one k-step; between(x) follows MFMA x
            constexpr int ks = decltype(ks_tag)::value;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    mfma_tied(acc[i][j], bfr[ks][j], af[ks][i]);     // transposed: lane = row, 4 columns
                    between(i * TN + j);
                }
        };
#pragma unroll
        for (int r = 0; r < NR; ++r) fetch_one(0, k0, r);
        int kt = 0;
        for (; kt + 2 < KT; ++kt) {                            // tile kt+1 is in flight or landed
            phase(k0, [&](int x) {
                if (x % 2 == 0 && x / 2 < NR) fetch_one(kt, k1, x / 2);
                if (x % 2 == 1 && x / 2 < A_INSTR) issue_load(kt + 2, 0, x / 2);
            });
            wait_loads_and_barrier<A_INSTR>();
            phase(k1, [&](int x) {
                if (x % 2 == 0 && x / 2 < B_INSTR) issue_load(kt + 2, 0, A_INSTR + x / 2);
                if (x % 2 == 1 && x / 2 < NR) fetch_one(kt + 1, k0, x / 2);
            });
        }
        for (; kt + 1 < KT; ++kt) {                            // the last tiles but one: nothing left to load
            phase(k0, [&](int x) { if (x % 2 == 0 && x / 2 < NR) fetch_one(kt, k1, x / 2); });
            wait_loads_and_barrier<0>();
            phase(k1, [&](int x) { if (x % 2 == 1 && x / 2 < NR) fetch_one(kt + 1, k0, x / 2); });
        }
        phase(k0, [&](int x) { if (x % 2 == 0 && x / 2 < NR) fetch_one(KT - 1, k1, x / 2); });
        phase(k1, [&](int) {});
        mfma_drain();
    } else if constexpr (PIPE) {
        auto fetch = [&](int kt, auto ks_tag) { fetch_into(kt, ks_tag, ks_tag); };   // k-step ks -> register set ks
        fetch(0, k0);
        for (int kt = 0; kt + 1 < KT; ++kt) {              // straight-line body: the last tile is peeled
            fetch(kt, k1);
            __builtin_amdgcn_sched_barrier(0);             // reads stay ahead of the MFMAs they overlap with
            mfmas(k0);
            __builtin_amdgcn_sched_barrier(0);
            tile_ready(kt + 1);
            fetch(kt + 1, k0);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(k1);
            __builtin_amdgcn_sched_barrier(0);
        }
        fetch(KT - 1, k1);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(k0);
        mfmas(k1);
    } else {
        for (int kt = 0; kt < KT; ++kt) {
            if (kt > 0) tile_ready(kt);
            fetch_into(kt, k0, k0);
            mfmas(k0);
            fetch_into(kt, k0, k1);
            mfmas(k0);
        }
    }

    if constexpr (SOLO) {
        __syncthreads();                                   // everyone is done with the tile buffers
        // The thread index computed again (the lane number from the execution mask, so that the compiler cannot
        // tell it is tid): otherwise everything the epilogue derives from it is computed once, ahead of the tile
        // loop, and kept in registers across the main loop, which has none to spare.
        int tid_e = wave * 64 + lane_id_again();
        if constexpr (SPLITK) {
            const int tile_sk = ((int)blockIdx.x & 7) * (total >> 3) + ((int)blockIdx.x >> 4);
            uint32_t use;
            if (!splitk_combine<TM, TN, NW * 64>(p, acc, tile_sk, tid_e, smem, use)) return;
            tid_e = wave * 64 + lane_id_again();
            gemm_epilogue_tile<BM, NW * 64, TM, TN, WTN, false, BN_OUT, false, true>(
                p, acc, smem, tid_e, m0, wm0, wn0, nloc0, seg, seg_rows,
                (const f32x4 *)p.sk_partial + (size_t)tile_sk * (TM * TN * NW * 64) + tid_e, p.sk_sync + 2 * tile_sk + 1, use);
            return;
        }
        if constexpr (ROPE)
            gemm_epilogue_tile_rope<BM, NW * 64, TM, TN, WTN, BN>(p, acc, smem, tid_e, m0, wm0, wn0, nloc0 >> 1, seg, seg_rows);
        else
            // only the 192-column tile takes GELU launches: with more accumulator blocks the compiler no longer
            // unrolls the (long) activation code and would index the accumulators through memory
            gemm_epilogue_tile<BM, NW * 64, TM, TN, WTN, SWIGLU, BN_OUT, TM * TN <= 48>(p, acc, smem, tid_e, m0, wm0, wn0, nloc0, seg, seg_rows);
    } else {
        __syncthreads();                                   // everyone is done with the tile buffers
        gemm_epilogue<TM, TN, WTN, SWIGLU>(p, acc, smem, wave, lane, m0, wm0, wn0, nloc0, seg, seg_rows);
    }
    if (!PERSISTENT || pid + (int)gridDim.x >= total) break;
    __syncthreads();                                       // the staged tile has been read: the next tile may load
    }
}

// ---------------------------------------------------------------------------- ping-pong variant
// Same tiles, loads, swizzle and epilogue as gemm2_kernel, different schedule.  The 8 wavefronts form
// two groups of 4 (one wavefront of each group per SIMD).  Every K tile is handled in two phases
// separated by workgroup barriers: a MEMORY phase (issue the direct-to-LDS loads of a tile NST-1
// ahead, read this tile's MFMA operands from LDS into registers) and a COMPUTE phase (nothing but
// MFMAs).  Group 1 runs one phase behind group 0, so on every SIMD one wavefront is always in its
// compute phase: the matrix pipe never waits for LDS latency or for a barrier bubble.
template <int VM, bool LGKM>
__device__ __forceinline__ void phase_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    if (VM >= 0 && LGKM) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM < 0 ? 0 : VM) : "memory");
    else if (VM >= 0) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(VM < 0 ? 0 : VM) : "memory");
    else if (LGKM) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool SWIGLU>
__global__ __launch_bounds__(WM *WN * 64) void gemm3_kernel(Gemm2Params p) {
    constexpr int NW = WM * WN;
    static_assert(NW == 8, "two groups of four wavefronts");
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 16, TN = WTN / 16;
    constexpr int ROWB = BK * 2, RPI = 1024 / ROWB, CPR = ROWB / 16, KS = BK / 32;
    constexpr int A_INSTR = BM / RPI / NW, B_INSTR = BN / RPI / NW;
    constexpr int LPT = A_INSTR + B_INSTR;
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(NST >= 2 && NST <= 5 && (NST - 2) * LPT < 64, "pipeline depth");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split over the wavefronts");
    static_assert(WTN == 64 || WTN == 128, "epilogue assumes 64 or 128 columns per wavefront");
    static_assert(!SWIGLU || (WTN == 128 && (WTN / 2) % RPI == 0), "swiglu layout");
    static_assert(NW * 16 * (WTN + 4) * 4 <= NST * STAGE_BYTES, "epilogue staging must fit in the tile buffers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = wave >> 2;                                   // wavefronts w and w+4 share a SIMD
    const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

    const int total = p.tiles_m * p.tiles_n;
    int tile;
    {
        const int pid = blockIdx.x, xcd = pid & 7, idx = pid >> 3;
        const int base = total >> 3, rem = total & 7;
        tile = xcd * base + min(xcd, rem) + idx;
    }
    int tile_m, tile_n;
    tile_coords(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int seg = tile_n >= p.seg_tile0[2] ? 2 : tile_n >= p.seg_tile0[1] ? 1 : 0;
    const int m0 = tile_m * BM;
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    const int nloc0 = (tile_n - p.seg_tile0[seg]) * BN_OUT;
    const int seg_rows = p.seg_rows[seg];
    const int K = p.K;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.X), 0, p.x_bytes, 0x00020000);
    const uint32_t w_bytes = (uint32_t)((int64_t)seg_rows * K * 2);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.W[seg]), 0, w_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ru =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(SWIGLU ? p.Wup : p.W[seg]), 0, w_bytes, 0x00020000);

    auto swz = [](int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
    uint32_t a_off[A_INSTR], b_off[B_INSTR];
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
        const int row = wave * (BM / NW) + RPI * i + lane / CPR;
        const int c = (lane % CPR) ^ swz(row);
        const int gm = m0 + row;
        a_off[i] = gm < p.M ? (uint32_t)(map_row_near(p.xmap, p.seq_len, gm, m0 / p.seq_len) * p.ldx * 2) + c * 16 : OOB_OFF;
    }
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
        const int row = wave * (BN / NW) + RPI * i + lane / CPR;
        const int c = (lane % CPR) ^ swz(row);
        int col;
        if (SWIGLU) col = nloc0 + (row / WTN) * (WTN / 2) + (row % (WTN / 2));
        else col = nloc0 + row;
        b_off[i] = col < seg_rows ? (uint32_t)((int64_t)col * K * 2) + c * 16 : OOB_OFF;
    }
    auto issue_loads = [&](int kt) {
        const int stage = kt % NST;
        const uint32_t kb = (uint32_t)kt * ROWB;
        unsigned char *sa = smem + stage * STAGE_BYTES + wave * (BM / NW) * ROWB;
        unsigned char *sb = smem + stage * STAGE_BYTES + A_BYTES + wave * (BN / NW) * ROWB;
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) load16_to_lds(rx, sa + i * 1024, a_off[i] + kb);
#pragma unroll
        for (int i = 0; i < B_INSTR; ++i) {
            const int row0 = wave * (BN / NW) + RPI * i;
            const bool up = SWIGLU && ((row0 % WTN) >= WTN / 2);
            if (up) load16_to_lds(ru, sb + i * 1024, b_off[i] + kb);
            else load16_to_lds(rw, sb + i * 1024, b_off[i] + kb);
        }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int frow = lane & 15, fch = lane >> 4, fsw = swz(lane & 15);
    const int a_lane = (wm0 + frow) * ROWB, b_lane = A_BYTES + (wn0 + frow) * ROWB;
    const int KT = K / BK;

    // Barrier bookkeeping.  Global barrier 2t ends group 0's memory phase of tile t and group 1's
    // compute phase of tile t-1; barrier 2t+1 ends group 0's compute phase and group 1's memory phase of
    // tile t, and is the one before which every wavefront makes sure its own loads of tile t+1 have
    // landed (so the tile is complete when group 0 starts reading it).
    // "tile t+1 landed" = at most the loads of the younger tiles t+2 .. min(KT-1, t+NST-1) outstanding.
#define WAIT_NEXT_TILE_AND_BARRIER(t, LG)                                    \
    do {                                                                     \
        const int younger = max(0, min(NST - 2, KT - 2 - (t)));              \
        if (younger >= 3) phase_barrier<3 * LPT, LG>();                      \
        else if (younger == 2) phase_barrier<2 * LPT, LG>();                 \
        else if (younger == 1) phase_barrier<LPT, LG>();                     \
        else phase_barrier<0, LG>();                                         \
    } while (0)

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < KT) issue_loads(s);
    {   // tile 0 complete and visible to everyone
        const int younger = max(0, min(NST - 2, KT - 1));
        if (younger >= 3) phase_barrier<3 * LPT, false>();
        else if (younger == 2) phase_barrier<2 * LPT, false>();
        else if (younger == 1) phase_barrier<LPT, false>();
        else phase_barrier<0, false>();
    }
    // With two stages a tile must be requested a whole tile period before it is read, so group 1
    // issues its share during its compute phase (the same window in which group 0 issues in its
    // memory phase); with three or more stages both groups issue in their memory phase.
    if (NST == 2 && group == 1 && 1 < KT) issue_loads(1);
    if (group == 1) phase_barrier<-1, false>();                    // run one phase behind group 0

    for (int kt = 0; kt < KT; ++kt) {
        // ---- memory phase: refill the stage of tile kt-1 (everyone finished reading it one barrier
        // ago), fetch this tile's operands
        if ((NST > 2 || group == 0) && kt + NST - 1 < KT) issue_loads(kt + NST - 1);
        const unsigned char *st = smem + (kt % NST) * STAGE_BYTES;
        bf16x8 af[KS][TM], bfr[KS][TN];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int coff = ((4 * ks + fch) ^ fsw) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i) af[ks][i] = *(const bf16x8 *)(st + a_lane + i * 16 * ROWB + coff);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[ks][j] = *(const bf16x8 *)(st + b_lane + j * 16 * ROWB + coff);
        }
        if (group == 1) WAIT_NEXT_TILE_AND_BARRIER(kt, true);
        else phase_barrier<-1, true>();
        // ---- compute phase
        if (NST == 2 && group == 1 && kt + 2 < KT) issue_loads(kt + 2);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
        if (group == 0) WAIT_NEXT_TILE_AND_BARRIER(kt, false);
        else phase_barrier<-1, false>();
    }
#undef WAIT_NEXT_TILE_AND_BARRIER
    if (group == 0) phase_barrier<-1, false>();                    // group 1 is one barrier ahead in count

    __syncthreads();
    gemm_epilogue<TM, TN, WTN, SWIGLU>(p, acc, smem, wave, lane, m0, wm0, wn0, nloc0, seg, seg_rows);
}

static int cu_count() {                                   // of the current device
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    return n;
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool SWIGLU, bool PINGPONG = false, bool ROPE = false,
          bool SPLITK = false>
static int32_t launch_cfg2(const GemmArgs &a, hipStream_t s) {
    Gemm2Params p;
    p.sk_partial = a.sk_partial; p.sk_sync = a.sk_sync;
    p.rope_table = a.rope_table; p.rope_cols = a.rope_cols; p.rope_lh = 0;
    if (ROPE) {
        while ((2 << p.rope_lh) < a.rope_head_dim) ++p.rope_lh;
        if ((uintptr_t)a.rope_table % 16) return CASCADE_EINVAL;
    }
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    int col0 = 0, tile0 = 0;
    for (int i = 0; i < 3; ++i) {
        int end = a.seg_end[i];
        int rows = std::max(0, end - col0);
        p.W[i] = (const bf16_t *)a.W[i];
        p.bias[i] = (const bf16_t *)a.bias[i];
        p.seg_rows[i] = rows;
        p.seg_col0[i] = col0;
        p.seg_tile0[i] = rows ? tile0 : INT32_MAX;
        tile0 += (rows + BN_OUT - 1) / BN_OUT;
        col0 = std::max(col0, end);
        if ((int64_t)rows * a.K * 2 >= (int64_t)OOB_OFF) return CASCADE_EUNSUPPORTED;
    }
    if (p.seg_tile0[0] == INT32_MAX) return CASCADE_ESHAPE;
    p.X = (const bf16_t *)a.X; p.Wup = (const bf16_t *)a.W_up; p.residual = (const bf16_t *)a.residual;
    p.Y = (bf16_t *)a.Y;
    p.M = a.M; p.K = a.K;
    p.tiles_m = (a.M + BM - 1) / BM; p.tiles_n = tile0;
    p.ldx = a.ldx; p.ldy = a.ldy; p.ldres = a.ldres;
    p.xmap = a.xmap.map; p.ymap = a.ymap.map; p.rmap = a.rmap.map;
    p.seq_len = a.xmap.map ? a.xmap.seq_len : a.ymap.map ? a.ymap.seq_len : a.rmap.map ? a.rmap.seq_len : 1;
    p.flags = a.epilogue;
    int64_t xb = (int64_t)a.M * a.ldx * 2;
    if (xb >= (int64_t)OOB_OFF) return CASCADE_EUNSUPPORTED;
    p.x_bytes = (uint32_t)xb;
    constexpr int LOAD_ROWS = 1024 / (BK * 2) * WM * WN;                  // B rows loaded per pass of all wavefronts
    constexpr int BNP = PINGPONG ? BN : (BN + LOAD_ROWS - 1) / LOAD_ROWS * LOAD_ROWS;
    constexpr size_t lds_loop = (size_t)NST * (BM + BNP) * BK * 2;
    constexpr size_t lds_solo = (size_t)(3 * BM + 2 * BNP) * BK * 2;            // three A stages, two B stages
    constexpr size_t lds = (!PINGPONG && WM * WN == 4) ? std::max(lds_solo, (size_t)EpiTile<BN_OUT>::bytes(BM)) : lds_loop;
    static_assert(lds <= 160 * 1024, "tile buffers exceed the LDS of a CU");
    const void *kern;
    if constexpr (PINGPONG) kern = (const void *)gemm3_kernel<BM, BN, WM, WN, BK, NST, SWIGLU>;
    else kern = (const void *)gemm2_kernel<BM, BN, WM, WN, BK, NST, SWIGLU, ROPE, SPLITK>;
    static std::atomic<uint64_t> lds_ready{0};                 // one per instantiation of this launcher
    CASCADE_HIP_TRY(ensure_dynamic_lds(kern, (int)lds, lds_ready));
    int64_t total = (int64_t)p.tiles_m * p.tiles_n;
    if (total > INT32_MAX) return CASCADE_EUNSUPPORTED;
    if (SPLITK) {                                              // what the kernel's tile mapping and scratch indexing assume
        if (total % 8 || total > GEMM_SPLITK_MAX_TILES || a.K % (2 * BK) || a.K / BK / 2 < 2) return CASCADE_EINVAL;
        if (!a.sk_partial || !a.sk_sync || a.sk_partial_bytes < (size_t)total * BM * BN * 4) return CASCADE_EWORKSPACE;
        if (((uintptr_t)a.sk_partial % 16) || ((uintptr_t)a.sk_sync % 4)) return CASCADE_EINVAL;
    }
    void *args[] = {&p};
    unsigned grid = (unsigned)(SPLITK ? 2 * total : total);
    if (!PINGPONG && !SPLITK && WM * WN == 4) {                 // persistent workgroups, one per CU, 8 | grid
        const int64_t per_round = cu_count() / 8 * 8;
        if (per_round >= 8 && total > per_round) grid = (unsigned)per_round;
    }
    CASCADE_HIP_TRY(hipLaunchKernel(kern, dim3(grid), dim3(WM * WN * 64), args, lds, s));
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}

static bool v2_eligible(const GemmArgs &a) {
    if (a.K % 64 != 0 || a.K < 64 || a.ldx % 8 != 0 || a.ldy % 4 != 0 || ((a.epilogue & CASCADE_EPI_RESIDUAL) && a.ldres % 4 != 0))
        return false;
    if (((uintptr_t)a.Y | (uintptr_t)a.residual | (uintptr_t)a.bias[0] | (uintptr_t)a.bias[1] | (uintptr_t)a.bias[2]) % 8)
        return false;                                                // 8-byte pieces of output, residual and bias
    for (int i = 0; i < 3; ++i)
        if (a.seg_end[i] % 4) return false;                         // 4-column store chunks stay inside a segment
    return true;
}

// Whether this launch (a.rope_head_dim and a.rope_cols set, a.rope_table not needed yet) can rotate its output
// in the epilogue: a plain projection (bias at most) whose segments hold whole heads of a power-of-two width.
bool gemm_bf16_rope_fusable(const GemmArgs &a) {
    if (a.dtype != CASCADE_BF16 || !v2_eligible(a)) return false;
    if (a.epilogue & ~CASCADE_EPI_BIAS) return false;
    const int hd = a.rope_head_dim;
    if (hd < 16 || hd > 256 || (hd & (hd - 1)) || a.rope_cols % hd) return false;
    int col0 = 0;
    for (int i = 0; i < 3; ++i) {
        const int rows = std::max(0, a.seg_end[i] - col0);
        if (rows % hd) return false;
        col0 = std::max(col0, a.seg_end[i]);
    }
    return true;
}

// Split reduction: 256 x 256 tiles would fill between a quarter and a half of the CUs (so two workgroups per
// tile fill them in one round), their number is a multiple of the 8 XCDs, and K is long enough to pay for the
// exchange (one segment of plain columns assumed: N is the output width).  Measured on MI355X at 2048 x 4096
// outputs against the 256 x 128 kernel on the same 256 CUs: the main loop gains 6 us at K = 4096 and 35-40 us at
// K = 14336, the exchange (256 KB written and read per tile, one L2 write-back and one invalidation per
// workgroup, the epilogue on half of the CUs) costs 15-20 us: 81 against 70 us and 195 against 205 us.
constexpr int GEMM_SPLITK_MIN_K = 8192;
size_t gemm_bf16_splitk_bytes(int32_t M, int32_t N, int32_t K) {
    if (M <= 0 || N <= 0 || K % 128 != 0 || K < GEMM_SPLITK_MIN_K) return 0;
    const int64_t tiles = (int64_t)((M + 255) / 256) * ((N + 255) / 256), cus = cu_count();
    if (tiles % 8 || tiles > GEMM_SPLITK_MAX_TILES || 2 * tiles > cus || 4 * tiles <= cus) return 0;
    return (size_t)tiles * 256 * 256 * 4;
}

// Returns CASCADE_EUNSUPPORTED when the shape is not eligible (the caller then uses the general kernel).
int32_t launch_gemm_bf16_v2(const GemmArgs &a, hipStream_t s) {
    if (!v2_eligible(a)) return a.rope_table ? CASCADE_EINVAL : CASCADE_EUNSUPPORTED;
    const bool swiglu = a.epilogue & CASCADE_EPI_SWIGLU;
    // Tile choice.  The cost of a launch is rounds of workgroups x columns per tile; candidates are
    // 256 rows x {256, 224, 192} columns (BK 64, two stages; the widths exist to fill whole rounds) and
    // 256 x 128 (three stages, ping-pong schedule).  The cheapest wins, the narrow one only by a margin.
    // SwiGLU always uses a wide tile (gate and up rows are interleaved inside it).  Measured on MI355X:
    // wide tiles 1.13 PFLOP/s on the FFN up GEMM with 8 wavefronts (1.06-1.08 for BK 32 with 4-5 stages),
    // 1.25-1.3 with one wavefront per SIMD; 256x128 ping-pong 1.10 against 1.04 PFLOP/s on FFN down.
    const int tiles_m = (a.M + 255) / 256;
    auto n_tiles = [&](int bn_out) {
        int64_t t = 0;
        int col0 = 0;
        for (int i = 0; i < 3; ++i) { int rows = std::max(0, a.seg_end[i] - col0); t += (rows + bn_out - 1) / bn_out; col0 = std::max(col0, a.seg_end[i]); }
        return t * tiles_m;
    };
    const int64_t cus = cu_count();
    auto cost = [&](int bne) { return ((n_tiles(swiglu ? bne / 2 : bne) + cus - 1) / cus) * bne; };
    const int64_t c256 = cost(256), c224 = cost(224), c192 = cost(192), c128 = cost(128);
    if (a.rope_table) {                  // rotary embedding in the epilogue: the one-wavefront kernels only
        if (!gemm_bf16_rope_fusable(a)) return CASCADE_EINVAL;
        const int64_t best = std::min(c192, std::min(c224, c256));
        if (c256 * 100 <= best * 104 && n_tiles(256) > cus) return launch_cfg2<256, 256, 2, 2, 64, 2, false, false, true>(a, s);
        if (c192 == best) return launch_cfg2<256, 192, 2, 2, 64, 2, false, false, true>(a, s);
        if (c224 == best) return launch_cfg2<256, 224, 4, 1, 64, 2, false, false, true>(a, s);
        return launch_cfg2<256, 256, 2, 2, 64, 2, false, false, true>(a, s);
    }
    if (swiglu) {
        if (c224 < c256) return launch_cfg2<256, 224, 4, 1, 64, 2, true, false>(a, s);
        return launch_cfg2<256, 256, 2, 2, 64, 2, true, false>(a, s);
    }
    {   // single-round launch of 256 x 128 tiles -> the same number of workgroups on 256 x 256 tiles, half of K each
        const bool gelu = a.epilogue & (CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH);
        const bool one_seg = a.seg_end[0] == a.N && a.seg_end[1] == a.N && a.seg_end[2] == a.N;
        const size_t need = (a.sk_partial && a.sk_sync && one_seg && !gelu) ? gemm_bf16_splitk_bytes(a.M, a.N, a.K) : 0;
        if (need && a.sk_partial_bytes >= need && (uintptr_t)a.sk_partial % 16 == 0)
            return launch_cfg2<256, 256, 2, 2, 64, 2, false, false, false, true>(a, s);
    }
    // the 256x128 kernel does ~15 % fewer flops per cycle than the wide ones: it has to be that much cheaper
    if (std::min(c192, std::min(c224, c256)) * 20 <= c128 * 23) {
        const int64_t best = std::min(c192, std::min(c224, c256));
        // 256 columns: the one-wavefront schedule when a CU works through several tiles of a long reduction and
        // the epilogue is light (its 256 accumulators leave the GELU code no registers); measured on
        // 8192 x 4096 x 4096 with residual 1.10 against 0.98 PFLOP/s, x 14336 1.27 against 1.14.  It goes before
        // the narrower tiles up to a 4 % higher cost: fewer tile-load instructions and operand reads per MFMA
        // (8192 x 32000 x 4096: 1.24 against 1.11 PFLOP/s for 192 columns at 1.6 % more rounds x width).
        const bool gelu = a.epilogue & (CASCADE_EPI_GELU_ERF | CASCADE_EPI_GELU_TANH);
        const bool solo256 = n_tiles(256) > cus && a.K >= 2048 && !gelu;
        if (c256 * 100 <= best * 104 && solo256) return launch_cfg2<256, 256, 2, 2, 64, 2, false, false>(a, s);
        // 192 and 224 columns: always the one-wavefront schedule, the narrowest cost first (2048 x 6144 x 4096 in
        // one round of 256 tiles: 86 us inside the layer against 100 us with 8 wavefronts)
        if (c192 == best) return launch_cfg2<256, 192, 2, 2, 64, 2, false, false>(a, s);
        if (c224 == best)
            return gelu ? launch_cfg2<256, 224, 4, 2, 64, 2, false, false>(a, s)     // 8 wavefronts
                        : launch_cfg2<256, 224, 2, 2, 64, 2, false, false>(a, s);
        return launch_cfg2<256, 256, 4, 2, 64, 2, false, false>(a, s);   // 8 wavefronts
    }
    // narrow GEMMs (N of a few hundred to a few thousand columns): 256x128 tiles, or 128x128 when even those
    // would leave half of the CUs without a workgroup (small-model o projection / FFN down)
    if (n_tiles(128) * 2 <= cus) return launch_cfg2<128, 128, 4, 2, 64, 3, false, true>(a, s);
    return launch_cfg2<256, 128, 4, 2, 64, 3, false, true>(a, s);
}
