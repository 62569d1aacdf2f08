// LoRA shrink: v[m, 0:r] = x[perm[m], :] . A_s[0:r, :]^T for every grouped row m whose slot s holds a
// rank-r adapter (paper Sec. 2.2: the first of the adapter's two low-rank matrices).
//
// Memory-bound: each adapter's A is streamed once per piece.  A work item is (piece, K chunk) and is
// owned by one wavefront: no LDS, no barriers.  Operands are loaded straight from global memory in
// the MFMA 32x32x16 bf16 lane layout.  Within a 64-wide K step lane (i, h) reads 64 contiguous bytes
// of row i at k0 + 32 h, and MFMA q of the step consumes bytes [16 q, 16 q + 16) of both halves; A and
// x use the same assignment, so the K order inside the step is permuted identically on both sides.
#include "lora_internal.hpp"

namespace lora {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ inline bf16x8 as_bf16x8(u32x4 v)
{
    return __builtin_bit_cast(bf16x8, v);
}

__device__ inline u32x4 load16(const uint16_t* p)
{
    return *reinterpret_cast<const u32x4*>(p);
}

constexpr int kShrinkThreads = 256;

__global__ __launch_bounds__(kShrinkThreads) void shrink_kernel(ShrinkArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    const int waves_per_block = kShrinkThreads / kWave;
    const int gw = blockIdx.x * waves_per_block + (threadIdx.x / kWave);
    const int stride = gridDim.x * waves_per_block;
    const int n_pieces = *a.dv.n_pieces;
    const int n_items = n_pieces * a.n_kc;
    const int K = a.K;
    const u32x4 zero = {0u, 0u, 0u, 0u};

    for (int item = gw; item < n_items; item += stride) {
        const int piece = item / a.n_kc;
        const int kc = item - piece * a.n_kc;
        const int slot = a.dv.piece_slot[piece];
        if (slot < 0) continue;
        const int r = a.dv.slot_rank[slot];
        if (r <= 0) continue;
        const int m_begin = a.dv.piece_start[piece];
        const int nrows = a.dv.piece_start[piece + 1] - m_begin;
        const int k_begin = kc * a.kc_len;
        int k_end = k_begin + a.kc_len;
        if (k_end > K) k_end = K;

        const bool x_ok = i < nrows;
        const uint16_t* xrow = a.x + (size_t)(x_ok ? a.dv.perm[m_begin + i] : 0) * K + h * 32;
        const uint16_t* As = a.dv.slots + (size_t)slot * a.dv.slot_stride + a.a_off;
        const bool a0_ok = i < r, a1_ok = (32 + i) < r;
        const uint16_t* arow0 = As + (size_t)(a0_ok ? i : 0) * K + h * 32;
        const uint16_t* arow1 = As + (size_t)(a1_ok ? 32 + i : 0) * K + h * 32;

        f32x16 acc0 = {0}, acc1 = {0};
        if (r <= 32) {
#pragma unroll 2
            for (int k0 = k_begin; k0 < k_end; k0 += kBK) {
                u32x4 xv[4], av[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    xv[q] = x_ok ? load16(xrow + k0 + q * 8) : zero;
                    av[q] = a0_ok ? load16(arow0 + k0 + q * 8) : zero;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av[q]), as_bf16x8(xv[q]), acc0, 0, 0, 0);
            }
        } else {
#pragma unroll 2
            for (int k0 = k_begin; k0 < k_end; k0 += kBK) {
                u32x4 xv[4], av[4], bv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    xv[q] = x_ok ? load16(xrow + k0 + q * 8) : zero;
                    av[q] = a0_ok ? load16(arow0 + k0 + q * 8) : zero;
                    bv[q] = a1_ok ? load16(arow1 + k0 + q * 8) : zero;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av[q]), as_bf16x8(xv[q]), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(bv[q]), as_bf16x8(xv[q]), acc1, 0, 0, 0);
                }
            }
        }

        // accumulator layout: column = i (grouped row m_begin + i), register v holds output row
        // j = 8 (v / 4) + 4 h + (v % 4)
        if (x_ok) {
            float* vrow = a.vpart + ((size_t)kc * a.dv.T + (size_t)(m_begin + i)) * a.dv.max_rank;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j = g * 8 + h * 4;
                if (j < r) {
                    f32x4 o = {acc0[g * 4 + 0], acc0[g * 4 + 1], acc0[g * 4 + 2], acc0[g * 4 + 3]};
                    *reinterpret_cast<f32x4*>(vrow + j) = o;
                }
            }
            if (r > 32) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int j = 32 + g * 8 + h * 4;
                    if (j < r) {
                        f32x4 o = {acc1[g * 4 + 0], acc1[g * 4 + 1], acc1[g * 4 + 2], acc1[g * 4 + 3]};
                        *reinterpret_cast<f32x4*>(vrow + j) = o;
                    }
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_shrink(const ShrinkArgs& a, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL(shrink_kernel, dim3(grid), dim3(kShrinkThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lora
