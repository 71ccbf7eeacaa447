// Measurement aid: sustained rate of v_mfma_f32_32x32x16_bf16 with register operands, the
// ceiling the MFMA conv kernels are priced against next to the published peak.
#include "conv_mfma_common.h"

__device__ __forceinline__ uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// bf16 pattern of a value that is roughly standard normal: sum of four uniform bytes, centred
__device__ __forceinline__ uint32_t probe_bf16(uint32_t h)
{
    const float v = ((float)((h & 255u) + ((h >> 8) & 255u) + ((h >> 16) & 255u) + (h >> 24)) - 510.0f) * (1.0f / 147.8f);
    return pack_bf16x2(v, 0.0f) & 0xFFFFu;
}

__global__ __launch_bounds__(256) void k_probe_mfma(int random_data, int iters, float* sink, unsigned long long* clk)
{
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t wa[4], wb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t s = (uint32_t)(((blockIdx.x * 256 + threadIdx.x) * 8 + i) * 4 + j);
            wa[j] = random_data ? (probe_bf16(probe_hash(4 * s)) | (probe_bf16(probe_hash(4 * s + 1)) << 16)) : 0x3F803F80u;
            wb[j] = random_data ? (probe_bf16(probe_hash(4 * s + 2)) | (probe_bf16(probe_hash(4 * s + 3)) << 16)) : 0x3F803F80u;
        }
        const uint4 va = make_uint4(wa[0], wa[1], wa[2], wa[3]), vb = make_uint4(wb[0], wb[1], wb[2], wb[3]);
        a[i] = *(const bf16x8*)&va; b[i] = *(const bf16x8*)&vb;
    }
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + u) & 7], acc[j], 0, 0, 0);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

extern "C" rh_status rh_probe_mfma(rh_ctx* ctx, int32_t random_data, double ms_target, double out[3])
{
    if (!ctx || !out) return RH_E_INVALID;
    if (!(ms_target > 0.0) || ms_target > 2000.0) RH_FAIL(ctx, RH_E_INVALID, "rh_probe_mfma: ms_target must be in (0, 2000]");
    hipDeviceProp_t prop;
    RH_HIP(ctx, hipGetDeviceProperties(&prop, ctx->device));
    const int wgs = prop.multiProcessorCount;                 // one 4-wave workgroup per CU: one wave per SIMD
    // 64 MFMAs of 32 cycles per iteration; the clock is not known in advance, take 2 GHz
    long long iters = (long long)(ms_target * 1e-3 * 2.0e9 / (64.0 * 32.0));
    if (iters < 1) iters = 1;
    if (iters > 0x3FFFFFFF) iters = 0x3FFFFFFF;
    float* sink = nullptr; unsigned long long* clk = nullptr;
    RH_HIP(ctx, hipMalloc((void**)&sink, (size_t)wgs * 256 * sizeof(float)));
    hipError_t e = hipMalloc((void**)&clk, 2 * sizeof(unsigned long long));
    if (e != hipSuccess) { (void)hipFree(sink); RH_HIP(ctx, e); }
    hipEvent_t t0, t1;
    (void)hipEventCreate(&t0); (void)hipEventCreate(&t1);
    hipLaunchKernelGGL(k_probe_mfma, dim3(wgs), dim3(256), 0, ctx->stream, random_data, 64, sink, clk);   // warm-up
    (void)hipEventRecord(t0, ctx->stream);
    hipLaunchKernelGGL(k_probe_mfma, dim3(wgs), dim3(256), 0, ctx->stream, random_data, (int)iters, sink, clk);
    (void)hipEventRecord(t1, ctx->stream);
    e = hipEventSynchronize(t1);
    float ms = 0.0f; unsigned long long hc[2] = {0, 1};
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
    if (e == hipSuccess) e = hipMemcpy(hc, clk, sizeof(hc), hipMemcpyDeviceToHost);
    (void)hipEventDestroy(t0); (void)hipEventDestroy(t1);
    (void)hipFree(sink); (void)hipFree(clk);
    RH_HIP(ctx, e);
    const double flop = (double)wgs * 4.0 * (double)iters * 64.0 * 2.0 * 32.0 * 32.0 * 16.0;
    out[0] = flop / ((double)ms * 1e-3) / 1e12;
    out[1] = hc[1] ? (double)hc[0] / (double)hc[1] * 0.1 : 0.0;
    out[2] = (double)hc[0] / ((double)iters * 64.0);
    return RH_OK;
}
