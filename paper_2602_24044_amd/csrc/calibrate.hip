// Ceiling probes: what this machine's HBM and matrix cores sustain, measured with the simplest kernels that can
// reach them.  A roofline fraction of the projection kernels (paper Sec. 5.2: the backbone term of the model
// latency is what the weight stream and the matrix cores allow) is read against the vendor's peak and, for
// insight, against these.  Not on the serving path.
#include "../../include/lora_mi355.h"
#include "lora_internal.hpp"

namespace lora {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Every workgroup reads a contiguous share of the buffer, 16 bytes per lane and load, kUnroll loads in flight per
// lane; one value per workgroup goes to the sink so that the loads stay.
constexpr int kStreamThreads = 512, kStreamUnroll = 8;
__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const u32x4* src, size_t n16, uint32_t* sink)
{
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per_wg;
    size_t end = begin + per_wg;
    if (end > n16) end = n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = begin + threadIdx.x;
    for (; i + (size_t)(kStreamUnroll - 1) * kStreamThreads < end; i += (size_t)kStreamUnroll * kStreamThreads) {
        u32x4 v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * kStreamThreads);
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) acc ^= v[u];
    }
    for (; i < end; i += kStreamThreads) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9e3779b9u) sink[blockIdx.x] = x;      // practically never: the value only has to be needed
}

// Back-to-back MFMAs on 16 independent accumulator blocks per wavefront, four wavefronts per workgroup; thread 0
// of every workgroup also reports the shader clock ticks and the 100 MHz wall clock ticks the loop took.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* sink, unsigned long long* ticks, int iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 7);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 7);
    }
    f32x16 acc[16];
#pragma unroll
    for (int n = 0; n < 16; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 16; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 16; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[n][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = c1 - c0;
        ticks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

}  // namespace
}  // namespace lora

extern "C" {

lora_status lora_calibrate_stream(const void* d_src, size_t bytes, int32_t workgroups, void* d_sink, void* stream)
{
    if (!d_src || !d_sink || bytes < 16 || workgroups < 1 || workgroups > 65536) return LORA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_src) & 15) return LORA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lora::stream_read_kernel, dim3(workgroups), dim3(lora::kStreamThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const lora::u32x4*>(d_src), bytes / 16,
                       static_cast<uint32_t*>(d_sink));
    return hipGetLastError() == hipSuccess ? LORA_OK : LORA_ERR_HIP;
}

lora_status lora_calibrate_mfma(int32_t workgroups, int32_t iters, void* d_sink, void* d_ticks, void* stream)
{
    if (!d_sink || !d_ticks || iters < 1 || workgroups < 1 || workgroups > 65536) return LORA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lora::mfma_loop_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float*>(d_sink), static_cast<unsigned long long*>(d_ticks), iters);
    return hipGetLastError() == hipSuccess ? LORA_OK : LORA_ERR_HIP;
}

}  // extern "C"
