// Yardstick kernels for roofline reports (not part of the denoising path): what this chip sustains for a plain
// streaming read, a plain copy, and a dense bf16 MFMA loop, measured by the benchmark harness next to the
// datasheet peaks.
#include "common.h"

namespace {

// dst[i] = src[i], 16 bytes per lane, grid-stride: the plain copy that HBM byte counters are calibrated with.
__global__ __launch_bounds__(256) void peak_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Streaming read: every workgroup reads one contiguous share of the buffer (the access pattern that reaches the
// highest cold-read rate on this chip) and folds it into one word so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void peak_read_kernel(const uint4 *__restrict__ src, unsigned *__restrict__ sink, size_t n16) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
    unsigned acc = 0;
    for (size_t i = lo + threadIdx.x; i < hi; i += 256) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) sink[blockIdx.x] = acc;     // practically never: keeps the loads alive
}

// Dense MFMA 32x32x16 bf16 on registers only: 4 independent accumulators per wavefront, `iters` rounds of 4.
__global__ __launch_bounds__(256) void peak_mfma_kernel(float *__restrict__ sink, int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
    }
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) c0[v] = c1[v] = c2[v] = c3[v] = 0.f;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" int dkv_peak_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst || bytes < 16 || bytes % 16) { dkv_set_error("copy yardstick: buffers of a multiple of 16 bytes"); return DKV_E_INVALID_ARG; }
    hipLaunchKernelGGL(peak_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

extern "C" int dkv_peak_read(const void *src, void *sink, size_t bytes, void *stream) {
    if (!src || !sink || bytes < 16 || bytes % 16) { dkv_set_error("read yardstick: a buffer of a multiple of 16 bytes and a sink"); return DKV_E_INVALID_ARG; }
    hipLaunchKernelGGL(peak_read_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<unsigned *>(sink), bytes / 16);
    DKV_LAUNCH_CHECK();
    return DKV_OK;
}

extern "C" int dkv_peak_mfma(void *sink, int32_t iters, double *flops, void *stream) {
    if (!sink || iters < 1 || !flops) { dkv_set_error("mfma yardstick: sink, iteration count and flops output"); return DKV_E_INVALID_ARG; }
    const int blocks = 256 * 8;       // 8 workgroups of 4 wavefronts per compute unit
    hipLaunchKernelGGL(peak_mfma_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float *>(sink), iters);
    DKV_LAUNCH_CHECK();
    *flops = (double)blocks * 4 /* wavefronts */ * iters * 4.0 * (2.0 * 32 * 32 * 16);
    return DKV_OK;
}
