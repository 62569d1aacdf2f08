// Stand-alone LoRA shrink launch (used ahead of the fused GEMM; the split-K GEMM runs the same work
// loop inside its own workgroups).  Memory-bound; no LDS, no barriers.
#include "device_common.hpp"

namespace lora {
namespace {

constexpr int kShrinkThreads = 256;

__global__ __launch_bounds__(kShrinkThreads) void shrink_kernel(ShrinkArgs a)
{
    const int waves_per_block = kShrinkThreads / kWave;
    shrink_wave_items(a, blockIdx.x * waves_per_block + (int)(threadIdx.x / kWave), gridDim.x * waves_per_block);
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs& a, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL(shrink_kernel, dim3(grid), dim3(kShrinkThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lora
