// Peak probes for MI355X (gfx950): plain streaming kernels and an fp32 MFMA loop.
// They are not part of the convolution path: the benchmark quotes what they reach next
// to the published peaks, and the copy kernel of known size calibrates the profiler's
// FETCH_SIZE / WRITE_SIZE counters.
#include <hip/hip_runtime.h>

typedef float floatx16 __attribute__((ext_vector_type(16)));

#define PROBE_API extern "C" __attribute__((visibility("default")))

__global__ __launch_bounds__(256) void probe_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                         size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_fill_kernel(float4* __restrict__ dst, size_t n4, float v)
{
    const float4 f = make_float4(v, v, v, v);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) dst[i] = f;
}

__global__ __launch_bounds__(256) void probe_read_kernel(const float4* __restrict__ src, float* __restrict__ out,
                                                         size_t n4)
{
    float s = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        const float4 v = src[i];
        s += v.x + v.y + v.z + v.w;
    }
    if (s == 123.456f) out[0] = s;  // keeps the loads alive without a store in practice
}

// 4 independent accumulator chains per wave, `iters` rounds of 4 MFMAs each.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters, float a, float b)
{
    floatx16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
    for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
    if (s == 123.456f) out[threadIdx.x] = s;
}

// bytes must be a multiple of 16; both pointers device memory, 16-byte aligned.
PROBE_API int dwm_probe_copy(const void* src_dev, void* dst_dev, size_t bytes, int blocks, void* stream)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const float4*)src_dev, (float4*)dst_dev, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

PROBE_API int dwm_probe_fill(void* dst_dev, size_t bytes, int blocks, void* stream)
{
    hipLaunchKernelGGL(probe_fill_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (float4*)dst_dev,
                       bytes / 16, 1.0f);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

PROBE_API int dwm_probe_read(const void* src_dev, void* out_dev, size_t bytes, int blocks, void* stream)
{
    hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const float4*)src_dev,
                       (float*)out_dev, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// Launches blocks x 4 waves; total flops = blocks * 4 * iters * 4 * 4096.
PROBE_API int dwm_probe_mfma(void* out_dev, int blocks, int iters, void* stream)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (float*)out_dev, iters,
                       1.0f, 0.5f);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}
