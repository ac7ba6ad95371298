// fp32 shard GEMM: Y[rows] = epilogue(X[rows] W^T).  Plain FMA arithmetic (no reduced-precision
// matrix path) so the result stays within 1e-5 of a float64 reference.  Used for the fp32
// configuration, which is latency-bound; the tile is small and simple on purpose.
#include "common.h"
#include "device_utils.h"
#include "epilogue.h"

#define F32_BM 64
#define F32_BN 64
#define F32_BK 16

template <bool SWIGLU>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ X, WeightSegs segs,
                                                       const float *__restrict__ Wup,
                                                       const float *__restrict__ residual, float *__restrict__ Y,
                                                       int M, int N, int K, int64_t ldx, int64_t ldy, int64_t ldres,
                                                       const int32_t *xmap, const int32_t *ymap,
                                                       const int32_t *rmap, int seq_len, int flags) {
    __shared__ float As[F32_BK][F32_BM + 1];
    __shared__ float Bs[F32_BK][F32_BN + 1];
    __shared__ float Us[SWIGLU ? F32_BK : 1][F32_BN + 1];
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
    const int m0 = blockIdx.y * F32_BM, n0 = blockIdx.x * F32_BN;

    // each thread stages 4 elements of A and of B per k-tile: element id = t + 256 i -> (row, kk)
    const float *arow[4];
    const float *brow[4];
    const float *urow[4];
    int lrow[4], lk[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int id = t + 256 * i;
        lrow[i] = id >> 4;
        lk[i] = id & 15;
        int gm = m0 + lrow[i], gn = n0 + lrow[i];
        arow[i] = gm < M ? X + map_row(xmap, seq_len, gm) * ldx : nullptr;
        brow[i] = gn < N ? weight_row<float>(segs, gn, K) : nullptr;
        urow[i] = (SWIGLU && gn < N) ? Wup + (int64_t)gn * K : nullptr;
    }
    float acc[4][4] = {};
    float acc2[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += F32_BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int k = k0 + lk[i];
            As[lk[i]][lrow[i]] = (arow[i] && k < K) ? arow[i][k] : 0.f;
            Bs[lk[i]][lrow[i]] = (brow[i] && k < K) ? brow[i][k] : 0.f;
            if (SWIGLU) Us[lk[i]][lrow[i]] = (urow[i] && k < K) ? urow[i][k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F32_BK; ++kk) {
            float a[4], b[4], u[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[kk][ty * 4 + i];
                b[i] = Bs[kk][tx * 4 + i];
                if (SWIGLU) u[i] = Us[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                    if (SWIGLU) acc2[i][j] = fmaf(a[i], u[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
        int64_t yr = map_row(ymap, seq_len, gm);
        int64_t rr = (flags & CASCADE_EPI_RESIDUAL) ? map_row(rmap, seq_len, gm) : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (flags & CASCADE_EPI_BIAS) v += bias_at<float>(segs, gn);
            if (SWIGLU) v = silu_f(v) * acc2[i][j];
            else v = apply_act(v, flags);
            if (flags & CASCADE_EPI_RESIDUAL) v += residual[rr * ldres + gn];
            Y[yr * ldy + gn] = v;
        }
    }
}

int32_t launch_gemm_f32(const GemmArgs &a, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return CASCADE_OK;
    WeightSegs segs;
    for (int i = 0; i < 3; ++i) { segs.w[i] = a.W[i]; segs.bias[i] = a.bias[i]; segs.end[i] = a.seg_end[i]; }
    dim3 grid((a.N + F32_BN - 1) / F32_BN, (a.M + F32_BM - 1) / F32_BM);
    if (grid.y > 65535) return CASCADE_EUNSUPPORTED;
    const int seq = a.xmap.map ? a.xmap.seq_len : a.ymap.map ? a.ymap.seq_len : a.rmap.seq_len;
    if (a.epilogue & CASCADE_EPI_SWIGLU)
        hipLaunchKernelGGL(gemm_f32_kernel<true>, grid, dim3(256), 0, s, (const float *)a.X, segs,
                           (const float *)a.W_up, (const float *)a.residual, (float *)a.Y, a.M, a.N, a.K, a.ldx,
                           a.ldy, a.ldres, a.xmap.map, a.ymap.map, a.rmap.map, seq, a.epilogue);
    else
        hipLaunchKernelGGL(gemm_f32_kernel<false>, grid, dim3(256), 0, s, (const float *)a.X, segs,
                           (const float *)a.W_up, (const float *)a.residual, (float *)a.Y, a.M, a.N, a.K, a.ldx,
                           a.ldy, a.ldres, a.xmap.map, a.ymap.map, a.rmap.map, seq, a.epilogue);
    CASCADE_HIP_TRY(hipGetLastError());
    return CASCADE_OK;
}
