// Peak probes for MI355X (gfx950): plain streaming kernels and an fp32 MFMA loop.
// They are not part of the convolution path: the benchmark quotes what they reach next
// to the published peaks, and the copy kernel of known size calibrates the profiler's
// FETCH_SIZE / WRITE_SIZE counters.
#include <hip/hip_runtime.h>

#include <cstdint>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

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

// ---------------------------------------------------------------------------------
// Operand-delivery probe: the instruction mix of one chunk of a 16-bit contraction workgroup (eight
// waves, two per SIMD), each ingredient alone or together.  Per iteration a wave issues NM MFMAs
// (32x32x16, one dependent chain), NL LDS reads of 1 KB (ds_read_b128) and ND global->LDS DMA
// instructions of 1 KB; at most `RING - 1` iterations of DMA are in flight; BAR = a workgroup barrier
// per iteration.  DMA sources: all but the last instruction of an iteration read a region every
// workgroup shares (`shared_mask` + 1 bytes, walked in step: L2 hits); the last reads a stream private
// to a pair of workgroups that sit on the same XCD (`pair_stride` bytes apart, 0 = shared region as
// well).  Every address is masked into the source buffer, which must hold 2^26 + 2^31 + 2^20 bytes.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void probe_dma16(const void* base_uniform, uint32_t lane_byte_offset, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_byte_offset), "s"(base_uniform), "s"(lds_addr)
                 : "memory");
}

template <int NM, int NL, int ND, int BAR, int RING>
__global__ __launch_bounds__(512) void probe_mix_kernel(const unsigned char* __restrict__ src, uint32_t* __restrict__ out,
                                                        int iters, uint32_t pair_stride, uint32_t shared_mask)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char sm[];  // 64 KB read area + RING * 8 * ND KB of DMA targets
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 16384; i += 512) reinterpret_cast<uint32_t*>(sm)[i] = i;
    __syncthreads();
    floatx16 acc;
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    halfx8 a, b;
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(lane * 0.01f + e);
        b[e] = (_Float16)(e - lane * 0.02f);
    }
    uintx4 r[8];
    for (int u = 0; u < 8; ++u) r[u] = uintx4{0, 0, 0, 0};
    const uint32_t lds0 = (uint32_t)(uintptr_t)sm;
    const uint32_t addr = lds0 + (uint32_t)(wave * 8192 + lane * 16);
    const uint32_t pair = (blockIdx.x & 7) + 8 * (blockIdx.x >> 4);  // blocks b and b + 8 share an XCD
    for (int it = 0; it < iters; ++it) {
        if (ND > 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(ND * (RING - 1)) : "memory");
        if (BAR) __syncthreads();
        const unsigned char* p = src + (((uint32_t)it * (uint32_t)(8 * ND * 1024)) & shared_mask);
        const unsigned char* q = src + (1u << 26) + ((pair * pair_stride + (uint32_t)it * 8192u) & ((1u << 31) - 1));
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            const uint32_t dst = lds0 + 65536u + (uint32_t)((((it % RING) * 8 + wave) * ND + d) * 1024);
            if (d == ND - 1 && pair_stride) probe_dma16(q, (uint32_t)(wave * 1024 + lane * 16), dst);
            else probe_dma16(p, (uint32_t)((wave * ND + d) * 1024 + lane * 16), dst);
        }
#pragma unroll
        for (int m = 0; m < (NM > NL ? NM : NL); ++m) {
            if (m < NL) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r[m & 7]) : "v"(addr), "n"((m & 7) * 1024));
            if (m < NM) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint32_t s = 0;
    for (int u = 0; u < 8; ++u) s ^= r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
    float f = 0;
    for (int e = 0; e < 16; ++e) f += acc[e];
    out[blockIdx.x * 512 + tid] = s ^ __float_as_uint(f);
}

template <int NM, int NL, int ND, int BAR, int RING>
static int probe_mix_launch(const void* src, void* out, int iters, int blocks, uint32_t pair_stride, uint32_t shared_mask, hipStream_t st)
{
    constexpr int lds = 65536 + RING * 8 * (ND > 0 ? ND : 1) * 1024;
    static_assert(lds <= 160 * 1024, "LDS");
    auto kern = probe_mix_kernel<NM, NL, ND, BAR, RING>;
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return 1;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), lds, st, (const unsigned char*)src, (uint32_t*)out, iters,
                       pair_stride, shared_mask);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// mode: 0 MFMAs only (4 per wave and iteration), 1 LDS reads only (8 KB per wave), 2 DMA only (3 KB per wave),
// 3 all three with a barrier, 4 all three with a ring of four iterations.  src_dev: 2^26 + 2^31 + 2^20 bytes;
// out_dev: blocks * 512 words; blocks <= 256 (one workgroup per CU).  pair_stride and shared_mask as above
// (shared_mask + 1 a power of two <= 2^26, pair_stride <= 2^24: 128 streams inside 2^31 bytes).
PROBE_API int dwm_probe_mix(const void* src_dev, void* out_dev, int mode, int iters, int blocks, unsigned pair_stride,
                            unsigned shared_mask, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (blocks < 1 || blocks > 256 || iters < 1 || (shared_mask & (shared_mask + 1)) != 0 || shared_mask >= (1u << 26) ||
        pair_stride > (1u << 24))
        return 1;
    switch (mode) {
        case 0: return probe_mix_launch<4, 0, 0, 0, 2>(src_dev, out_dev, iters, blocks, pair_stride, shared_mask, st);
        case 1: return probe_mix_launch<0, 8, 0, 0, 2>(src_dev, out_dev, iters, blocks, pair_stride, shared_mask, st);
        case 2: return probe_mix_launch<0, 0, 3, 0, 2>(src_dev, out_dev, iters, blocks, pair_stride, shared_mask, st);
        case 3: return probe_mix_launch<4, 8, 3, 1, 2>(src_dev, out_dev, iters, blocks, pair_stride, shared_mask, st);
        case 4: return probe_mix_launch<4, 8, 3, 1, 4>(src_dev, out_dev, iters, blocks, pair_stride, shared_mask, st);
        default: return 1;
    }
}
