// Measured ceilings for the roofline figures: the rate the MFMA pipe sustains on this device with
// operands held in registers, and with operands re-read from LDS at the shard GEMM's ratio (12
// 16-byte reads per 32 MFMAs).  Random bf16 operands: the sustained clock, and with it the rate,
// depends on how many bits toggle.  Not part of the layer path.
#include <hip/hip_runtime.h>
#include "common.h"
#include "device_utils.h"

template <bool LDS_OPERANDS>
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(float *sink, int iters) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[49152];
    const int lane = threadIdx.x & 63;
    unsigned h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
    auto rnd = [&]() { h ^= h << 13; h ^= h >> 17; h ^= h << 5; return ((int)(h & 0xffff) - 32768) * (1.0f / 32768.f); };
    bf16x8 a[4], b[8];
    for (int i = 0; i < 4; ++i) for (int x = 0; x < 8; ++x) a[i][x] = (bf16_t)rnd();
    for (int i = 0; i < 8; ++i) for (int x = 0; x < 8; ++x) b[i][x] = (bf16_t)(0.05f * rnd());
    for (int i = threadIdx.x; i < 49152 / 2; i += 512) ((bf16_t *)lds)[i] = (bf16_t)(0.05f * rnd());
    __syncthreads();
    f32x4 acc[4][8];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
        if (LDS_OPERANDS) {                                // 12 KB per wavefront per 32 MFMAs, conflict-free
            const unsigned char *st = lds + ((it & 3) << 12) + lane * 16;
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *(const bf16x8 *)(st + i * 1024);
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = *(const bf16x8 *)(st + 16384 + j * 1024 + (j >= 4 ? 12288 : 0));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 8; ++j) for (int x = 0; x < 4; ++x) s += acc[i][j][x];
    if (s == 12345.678f) sink[0] = s;                      // keeps the accumulators alive
}

extern "C" int32_t cascade_mfma_ceiling(int32_t lds_operands, int32_t iters, float *tflops_out, void *stream) {
    if (!tflops_out || iters <= 0 || iters > (1 << 22)) return CASCADE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 0;
    CASCADE_HIP_TRY(hipGetDevice(&dev));
    CASCADE_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    float *sink = nullptr;
    CASCADE_HIP_TRY(hipMalloc((void **)&sink, 256));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t err = hipEventCreate(&e0);
    if (err == hipSuccess) err = hipEventCreate(&e1);
    float ms = 0.f;
    for (int rep = 0; rep < 2 && err == hipSuccess; ++rep) {         // first repetition warms the clocks up
        err = hipEventRecord(e0, s);
        if (err != hipSuccess) break;
        if (lds_operands) hipLaunchKernelGGL(mfma_ceiling_kernel<true>, dim3(cus), dim3(512), 0, s, sink, iters);
        else hipLaunchKernelGGL(mfma_ceiling_kernel<false>, dim3(cus), dim3(512), 0, s, sink, iters);
        err = hipGetLastError();
        if (err == hipSuccess) err = hipEventRecord(e1, s);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    CASCADE_HIP_TRY(err);
    // 32 MFMAs of 16x16x32 (16384 flop each) per iteration per wavefront, 8 wavefronts per workgroup
    *tflops_out = (float)(32.0 * 16384.0 * iters * 8.0 * cus / (ms * 1e-3) / 1e12);
    return CASCADE_OK;
}
