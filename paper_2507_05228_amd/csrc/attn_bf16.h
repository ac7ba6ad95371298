// Declarations shared by the bf16 attention kernels (partial attention, and fused attention for short
// shards: attn_bf16.hip; fused attention, software-pipelined: attn_bf16_fused.hip).
#pragma once
#include "common.h"
#include "device_utils.h"

#define KV_TILE 64
#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f
#define OOB_OFF 0x80000000u

typedef __attribute__((address_space(3))) void lds_void;
// Plan metadata is read-only for the kernel and indexed uniformly: reading it through the constant
// address space makes these scalar loads, which do not share a counter with the tile loads in flight.
typedef const __attribute__((address_space(4))) CascadeTile *tile_cptr;
typedef const __attribute__((address_space(4))) int32_t *int_cptr;

__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t r, unsigned char *lds, uint32_t voff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void *)lds, 16, voff, 0, 0, 0);
}
__device__ __forceinline__ void load4_to_lds(__amdgpu_buffer_rsrc_t r, unsigned char *lds, uint32_t voff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void *)lds, 4, voff, 0, 0, 0);
}

// max over the 4 lanes {l, l^16, l^32, l^48} with the gfx950 lane-swap instructions (no LDS traffic)
__device__ __forceinline__ float xor_max_16_32(float v) {
    typedef __attribute__((ext_vector_type(2))) unsigned u2;
    u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor_sum_16_32(float v) {
    typedef __attribute__((ext_vector_type(2))) unsigned u2;
    u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Workgroup barrier as inline assembly, optionally preceded by "all but the VM youngest vector-memory
// operations of this wavefront are complete" and "all LDS reads have returned".  (A compiler-generated
// barrier waits for vmcnt(0) and would drain the tile pipeline.)
template <int VM, bool LGKM>
__device__ __forceinline__ void phase_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    if (VM >= 0 && LGKM) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM < 0 ? 0 : VM) : "memory");
    else if (VM >= 0) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(VM < 0 ? 0 : VM) : "memory");
    else if (LGKM) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

struct AttnBf16Params {
    const bf16_t *q, *k, *vt;
    int64_t qs_b, qs_h, qs_n, ks_b, ks_h, ks_n, vts_b, vts_h;
    int32_t npad;
    uint32_t k_bytes, vt_bytes;      // extent of one (batch, kv head) slice, for the buffer resources
    const int32_t *q_rowmap;
    const CascadeTile *qtiles;
    const CascadeTile *kvtiles;      // ordered by smallest position: globally (fused) or inside each shard's range
    const int32_t *kv_shard_first;
    int32_t n_kvtiles;
    const int32_t *pos_packed;       // positions of the packed query rows
    const int32_t *pos_kv;           // positions of the key/value rows in the order of the kv tiles
    const int32_t *pos_kv_padded;    // the same, 64 per tile (at 64 * the tile's index), INT_MAX past a tile's end
    int32_t B, H, Hkv, N, S;
    float scale_log2;
    int32_t causal, fused, u_mode;
    float *m, *e, *u;
    bf16_t *o;
    int64_t o_ld;
    const int32_t *o_rowmap;
    int32_t hpb;          // heads per workgroup (1, 2 or 4)
    int32_t gy;           // (batch, kv head, head block) combinations: blockIdx.x = query tile * gy + combination
    // the same decomposition by multiplications (fused kernel): heads = kv heads x head blocks, rep = H / Hkv,
    // hblocks = rep / hpb, and the reciprocals of div_magic() for gy, heads and hblocks
    int32_t hpb_log2, rep, hblocks, heads;
    uint64_t gy_magic, heads_magic, hblocks_magic;
};

// floor(n / d) as a multiplication: magic = ceil(2^40 / d); exact while n d < 2^40 (and n / d < 2^23, so that the
// product stays inside 64 bits)
static inline uint64_t div_magic(uint32_t d) { return ((1ull << 40) + d - 1) / d; }
static inline bool div_magic_covers(uint64_t n_max, uint32_t d) { return n_max * d < (1ull << 40) && n_max / d < (1ull << 23); }
__host__ __device__ __forceinline__ uint32_t div_by_magic(uint32_t n, uint64_t magic) { return (uint32_t)(((uint64_t)n * magic) >> 40); }



// Fused attention, software-pipelined (attn_bf16_fused.hip).  The parameters are the ones the kernel of
// attn_bf16.hip takes; the query tiles are those of granule 256 / hpb rows.
// all_visible: no causal mask and no ragged key/value tile, i.e. no score needs a compare.
// split: the query tiles are 32-row tiles and each workgroup's two wavefront groups share one, every other
// key/value tile each (four heads per workgroup, masked kernel only).
int32_t launch_attn_fused(const AttnBf16Params &k, int head_dim, int n_qtiles, bool all_visible, bool split, hipStream_t s);
