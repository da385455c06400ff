// Roofline probes: what this GPU sustains on the two resources the library's kernels are bound by.
// They touch none of the method's arithmetic; the benchmark times them next to the real kernels so
// that fractions can be quoted against the measured rates as well as the published peaks.
#include "bf16_device.h"

namespace pevlm {

// Every wavefront issues v_mfma_f32_32x32x16_bf16 back to back on register operands (four
// independent accumulators); two 256-thread workgroups fit a compute unit, as in the attention
// kernel.  32768 floating-point operations per instruction per wavefront.
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(float *sink, int32_t iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        a[j] = (__bf16)(float)((threadIdx.x + j) & 7);
        b[j] = (__bf16)(float)((threadIdx.x * 3 + j) & 3);
    }
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    if (s == -1.f) sink[0] = s;  // never true: the accumulators only grow
}

// Streaming copy: a workgroup moves one contiguous 16 KB piece, 16 bytes per lane per access, four
// loads in flight per lane before the first store.
__global__ __launch_bounds__(256) void probe_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, int64_t n16)
{
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    uint4 r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (base + j * 256 < n16) r[j] = src[base + j * 256];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (base + j * 256 < n16) dst[base + j * 256] = r[j];
}

hipError_t launch_probe_mfma(float *sink, int32_t workgroups, int32_t iters, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, stream, sink, iters);
    return hipGetLastError();
}

hipError_t launch_probe_copy(void *dst, const void *src, int64_t bytes, hipStream_t stream)
{
    const int64_t n16 = bytes / 16;
    const int64_t blocks = (n16 + 1023) / 1024;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, (uint4 *)dst, (const uint4 *)src, n16);
    return hipGetLastError();
}

}  // namespace pevlm
