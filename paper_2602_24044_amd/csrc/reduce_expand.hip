// Split-K reduction fused with the LoRA expand and the output rounding:
//   out[perm[m], n] = bf16( sum_s part[s][m][n] + scale * sum_j v[m][j] B_slot[n][j] )
// (paper Sec. 2.2: the second low-rank matrix maps the adapter's activations back to the layer's
// output, where they are added to the backbone result).
//
// Memory-bound.  A work item is (piece, 1024-column chunk): the piece's rows all use one slot, so the
// chunk of B is read once per piece, 16 bytes per lane and contiguous across lanes; v (summed over
// the shrink's K chunks and scaled, fp32) is staged in LDS and broadcast.
#include "lora_internal.hpp"

namespace lora {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

constexpr int kRT = 256;          // threads
constexpr int kCols = kRT * 4;    // columns per work item
constexpr int kRowGroup = 8;

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__global__ __launch_bounds__(kRT) void reduce_expand_kernel(ReduceArgs a)
{
    __shared__ __attribute__((aligned(16))) float sV[kPieceRows][kMaxRank];
    const int tid = threadIdx.x;
    const int T = a.dv.T, N = a.N;
    const int n_pieces = *a.dv.n_pieces;
    const int n_items = n_pieces * a.n_chunks;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int piece = item / a.n_chunks;
        const int chunk = item - piece * a.n_chunks;
        const int slot = a.dv.piece_slot[piece];
        const int r = slot >= 0 ? a.dv.slot_rank[slot] : 0;
        const int m_begin = a.dv.piece_start[piece];
        const int nrows = a.dv.piece_start[piece + 1] - m_begin;
        const int n = chunk * kCols + tid * 4;
        const bool n_ok = n < N;

        if (r > 0) {
            const float sc = a.dv.slot_scale[slot];
            for (int e = tid; e < nrows * r; e += kRT) {
                const int row = e / r, j = e - row * r;
                float s = 0.f;
                for (int c = 0; c < a.n_kc; ++c)
                    s += a.vpart[((size_t)c * T + (m_begin + row)) * a.dv.max_rank + j];
                sV[row][j] = s * sc;
            }
        }
        __syncthreads();

        const uint16_t* Bs = a.dv.slots + (size_t)(slot >= 0 ? slot : 0) * a.dv.slot_stride + a.b_off
                             + (size_t)n * r;
        for (int row0 = 0; row0 < nrows; row0 += kRowGroup) {
            const int nr = (nrows - row0) < kRowGroup ? (nrows - row0) : kRowGroup;
            f32x4 acc[kRowGroup];
#pragma unroll
            for (int rr = 0; rr < kRowGroup; ++rr) {
                acc[rr] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (rr < nr && n_ok) {
                    const size_t m = (size_t)(m_begin + row0 + rr);
                    for (int s = 0; s < a.split_k; ++s)
                        acc[rr] += *reinterpret_cast<const f32x4*>(a.part + ((size_t)s * a.Mpad + m) * N + n);
                }
            }
            if (r > 0 && n_ok) {
                for (int jc = 0; jc < r; jc += 8) {
                    u32x4 b[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) b[q] = *reinterpret_cast<const u32x4*>(Bs + (size_t)q * r + jc);
#pragma unroll
                    for (int rr = 0; rr < kRowGroup; ++rr) {
                        if (rr < nr) {
                            const f32x4 v0 = *reinterpret_cast<const f32x4*>(&sV[row0 + rr][jc]);
                            const f32x4 v1 = *reinterpret_cast<const f32x4*>(&sV[row0 + rr][jc + 4]);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                float d = acc[rr][q];
                                d += v0[0] * bf16_lo(b[q][0]);
                                d += v0[1] * bf16_hi(b[q][0]);
                                d += v0[2] * bf16_lo(b[q][1]);
                                d += v0[3] * bf16_hi(b[q][1]);
                                d += v1[0] * bf16_lo(b[q][2]);
                                d += v1[1] * bf16_hi(b[q][2]);
                                d += v1[2] * bf16_lo(b[q][3]);
                                d += v1[3] * bf16_hi(b[q][3]);
                                acc[rr][q] = d;
                            }
                        }
                    }
                }
            }
            if (n_ok) {
#pragma unroll
                for (int rr = 0; rr < kRowGroup; ++rr) {
                    if (rr < nr) {
                        const int tok = a.dv.perm[m_begin + row0 + rr];
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[rr][e];
                        *reinterpret_cast<u32x2*>(a.out + (size_t)tok * N + n) = __builtin_bit_cast(u32x2, o);
                    }
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_reduce_expand(const ReduceArgs& a, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_expand_kernel, dim3(grid), dim3(kRT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lora
