// Split-K reduction fused with the LoRA expand and the output rounding:
//   out[perm[m], n] = bf16( sum_s part[s][m][n] + bias[n] + scale * sum_j v[m][j] B_slot(m)[n][j] )
// (paper Sec. 2.2: the second low-rank matrix maps the adapter's activations back to the layer's
// output, where they are added to the backbone result).
//
// Memory-bound.  One workgroup of four wavefronts owns a 32-row window of grouped rows and 128 output
// columns.  The window's shrink results are summed over the shrink's K chunks, scaled, rounded to bf16
// and parked in LDS once; each wavefront then sums the fp32 partial tiles of its 32 columns directly
// in MFMA accumulator layout and runs the expand as extra MFMA K steps, one pass per distinct slot in
// the window, reading that slot's B rows once.
#include "device_common.hpp"

namespace lora {
namespace {

constexpr int kRT = 256;
constexpr int kVStride = kMaxRank + 8;   // bf16 elements per LDS row: 144 bytes, conflict-free 16-byte reads

__global__ __launch_bounds__(kRT) void reduce_expand_kernel(ReduceArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t sV[kPieceRows * kVStride];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, h = lane >> 5;
    const int T = a.dv.T;                                             // stride of the shrink results
    const int m_end = a.m_end;
    const int n_win = (m_end - a.m_begin + kPieceRows - 1) / kPieceRows;   // windows counted from m_begin
    const int win = blockIdx.x % n_win, group = blockIdx.x / n_win;   // group: 128 packed columns
    // the slice (projection of a packed group) these columns belong to: slices start on multiples of 128
    int si = 0;
    for (int k = 1; k < a.g.n; ++k)
        if (group * 4 >= a.g.s[k].blk0) si = k;
    const Slice sl = pick_slice(a.g, si);
    const int N = sl.N;
    const int m = a.m_begin + win * kPieceRows + i;
    const bool m_ok = m < m_end;
    const int n_first = (group * 4 - sl.blk0) * 32 + wave * 32;       // column inside the slice

    // The kernel is a chain of memory round trips; everything whose address is known at the start is requested
    // at the start, oldest first what the next dependent load needs: this lane's row (slot, rank, token), the
    // rank and scale of the row this thread stages, then the partial tiles.
    const int my_slot[1] = {m_ok ? a.dv.row_loc[m] : -1};
    const int my_rank[1] = {m_ok ? a.dv.row_rank[m] : 0};
    const int my_tok = m_ok ? a.dv.perm[m] : 0;
    const int st_row = tid >> 3, st_seg = tid & 7;
    const int st_m = a.m_begin + win * kPieceRows + st_row;
    const bool st_on = st_m < m_end && st_seg * 8 < a.dv.max_rank;
    const int st_rank = st_on ? a.dv.row_rank[st_m] : 0;
    const float st_scale = st_on ? a.dv.row_scale[st_m] : 0.f;

    f32x16 acc[1];
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][v] = 0.f;
    // partial tiles are stored block by block in accumulator order (see the split-K GEMM): block
    // (window, n / 32) of split s is 1 KB-contiguous per register group, so these loads are fully
    // coalesced; four splits (16 independent 16-byte loads per lane) are kept in flight
    const int nblk = a.nblk;
    const int bn = group * 4 + wave;                                  // block in the packed partial matrix
    const bool cols_on = n_first < N;
    f32x4 p[4][4];
    auto load_splits = [&](int s0) {
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) {
            const int sp = (s0 + ds < a.split_k) ? s0 + ds : s0;
            const float* blk = a.part + (((size_t)sp * (a.Mpad / 32) + (size_t)win) * nblk + bn) * 1024;
#pragma unroll
            for (int g = 0; g < 4; ++g) p[ds][g] = *reinterpret_cast<const f32x4*>(blk + g * 256 + i * 8 + h * 4);
        }
    };
    auto add_splits = [&](int s0) {
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) {
            if (s0 + ds < a.split_k) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[0][g * 4 + e] += p[ds][g][e];
            }
        }
    };
    if (cols_on) load_splits(0);
    // bias of the backbone layer (null: none), this lane's 16 columns
    bf16x4 bias[4];
    const bool bias_on = sl.bias != nullptr;
    if (bias_on) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n_first + g * 8 + h * 4;
            bias[g] = __builtin_bit_cast(bf16x4, n < N ? *reinterpret_cast<const u32x2*>(sl.bias + n) : u32x2{0u, 0u});
        }
    }

    // the window's shrink results, thread -> (row, 8 ranks): requested behind the first partial tiles, for every
    // existing row whatever its rank (what lies beyond a row's rank was never written and is dropped below): the
    // loads then do not wait for the row's rank to arrive, one memory round trip less on the kernel's chain
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    if (st_on) {
#pragma unroll 4
        for (int c = 0; c < a.n_kc; ++c) {
            const float* vp = sl.vpart + ((size_t)c * T + st_m) * a.dv.max_rank + st_seg * 8;
            lo += *reinterpret_cast<const f32x4*>(vp);
            hi += *reinterpret_cast<const f32x4*>(vp + 4);
        }
    }

    if (cols_on) {
        add_splits(0);
        for (int s0 = 4; s0 < a.split_k; s0 += 4) {
            load_splits(s0);
            add_splits(s0);
        }
    }

    if (bias_on) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[0][g * 4 + e] += (float)bias[g][e];
    }

    // stage the scaled shrink results as bf16
    {
        u32x4 packed = {0u, 0u, 0u, 0u};
        if (st_on && st_seg * 8 < st_rank) {
            bf16x8 vb;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vb[e] = (__bf16)(lo[e] * st_scale);
                vb[4 + e] = (__bf16)(hi[e] * st_scale);
            }
            packed = __builtin_bit_cast(u32x4, vb);
        }
        *reinterpret_cast<u32x4*>(sV + st_row * kVStride + st_seg * 8) = packed;
    }
    __syncthreads();

    f32x16 accw[1][1] = {{acc[0]}};
    expand_windows<1, 1, 12>(accw, my_slot, my_rank, n_first, N, a.dv, sl.b_unit, sV);
    acc[0] = accw[0][0];

    if (m_ok) {
        uint16_t* orow = sl.out + (size_t)my_tok * N;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n_first + g * 8 + h * 4;
            if (n < N) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[0][g * 4 + e];
                *reinterpret_cast<u32x2*>(orow + n) = __builtin_bit_cast(u32x2, o);
            }
        }
    }
}

}  // namespace

hipError_t launch_reduce_expand(const ReduceArgs& a, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_expand_kernel, dim3(grid), dim3(kRT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lora
