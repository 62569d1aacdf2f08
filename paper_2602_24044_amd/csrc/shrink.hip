// Stand-alone LoRA shrink launch (used ahead of the fused GEMM; the split-K GEMM runs the same work
// loop inside its own workgroups).  Memory-bound.
#include "device_common.hpp"

namespace lora {
namespace {

constexpr int kShrinkThreads = 256;

__global__ __launch_bounds__(kShrinkThreads) void shrink_kernel(ShrinkArgs a)
{
    constexpr int NW = kShrinkThreads / kWave;
    __shared__ __attribute__((aligned(16))) float sRed[NW * kRedFloatsPerWave];
    const ShrinkPrefetch pf = shrink_prefetch(a, blockIdx.x);
    shrink_block_items<NW>(a, blockIdx.x, gridDim.x, pf.n_items, sRed, pf);
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs& a, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL(shrink_kernel, dim3(grid), dim3(kShrinkThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lora
