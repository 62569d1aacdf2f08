// What a GEMM wavefront does with its finished accumulators; shared by the GEMM kernels.
//   fused path: LoRA expand on the accumulators (paper Sec. 2.2: the adapter's activations are added to the
//               backbone layer's output), one bf16 rounding, rows scattered back to token order;
//   split path: fp32 partial tile for the reduce + expand kernel.
#pragma once

#include "device_common.hpp"

namespace lora {

// Fused path, wave tiles of at most two 32-row windows: what the epilogue needs from memory besides the B rows
// is fetched before the main loop and waits in registers, so that the tail of the kernel - which no other
// workgroup overlaps when the launch is a single round - holds one memory latency per (window, slot) pair
// instead of three per window.
template <int MB>
struct TilePrefetch {
    int slot[MB], rank[MB];          // this lane's row of each window
    float scale[MB];
    u32x4 v[MB][4];                  // this lane's shares of the windows' scaled shrink results (packed bf16)
};

template <int MB>
__device__ __forceinline__ void prefetch_windows(TilePrefetch<MB>& pf, const GemmArgs& a, const Slice& sl, int m_first)
{
    const int i = threadIdx.x & 31;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;
        const bool ok = m < a.m_end;
        pf.slot[mb] = ok ? a.dv.row_slot[m] : -1;
        pf.rank[mb] = ok ? a.dv.row_rank[m] : 0;
        pf.scale[mb] = ok ? a.dv.row_scale[m] : 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) pf.v[mb][q] = window_v_share(q, sl.vpart, a.n_kc, m_first + mb * 32, a.dv);
    }
}

// Epilogue of the fused path from prefetched window data.  ring: LDS free again (the caller has synchronised);
// this wave parks its MB windows at ring + wave * MB * kPieceRows * kVStageStride.
template <int MB, int NB>
__device__ __forceinline__ void finish_tile_prefetched(f32x16 (&acc)[MB][NB], const GemmArgs& a, const Slice& sl,
                                                       int m_first, int n_first, int wave, uint16_t* ring,
                                                       const TilePrefetch<MB>& pf)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    const int T = a.m_end, N = sl.N;
    bool any = false;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) any = any || __ballot(pf.slot[mb] >= 0 && pf.rank[mb] > 0) != 0;
    if (any) {                                                    // uniform over the wave
        uint16_t* sV = ring + wave * (MB * kPieceRows * kVStageStride);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q) park_v_share(sV + mb * kPieceRows * kVStageStride, q, pf.v[mb][q]);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        expand_windows<MB, NB, 4>(acc, pf.slot, pf.rank, n_first, N, a.dv, sl.b_off, sV);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;
        if (m < T) {
            uint16_t* orow = sl.out + (size_t)a.dv.perm[m] * N;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n_first + nb * 32 + g * 8 + h * 4;
                    if (n < N) {
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[mb][nb][g * 4 + e];
                        *reinterpret_cast<u32x2*>(orow + n) = __builtin_bit_cast(u32x2, o);
                    }
                }
        }
    }
}

// acc[mb][nb]: 32x32 blocks in "W-first" orientation (lane (i, h) holds grouped row m_first + 32 mb + i and
// output columns n_first + 32 nb + 8 g + 4 h + e in register 4 g + e); n_first is a column inside slice sl.
// ring: LDS no longer used by the main loop (the caller has synchronised); the fused path parks the scaled
// shrink results of one 32-row window at a time in this wave's piece of it.
template <int MB, int NB, bool FUSED>
__device__ __forceinline__ void finish_tile(f32x16 (&acc)[MB][NB], const GemmArgs& a, const Slice& sl, int m_first,
                                            int n_first, int split, int wave, uint16_t* ring)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    const int T = a.m_end, N = sl.N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;      // grouped row of this lane
        const bool m_ok = m < T;

        if (FUSED) {
            const int my_slot = m_ok ? a.dv.row_slot[m] : -1;
            const int my_rank = m_ok ? a.dv.row_rank[m] : 0;
            const float my_scale = m_ok ? a.dv.row_scale[m] : 0.f;
            if (__ballot(my_slot >= 0 && my_rank > 0)) {      // uniform over the wave
                uint16_t* sV = ring + wave * (kPieceRows * kVStageStride);
                stage_window_v(sV, sl.vpart, a.n_kc, m_first + mb * 32, a.dv);
                auto vfrag = [&](int k, bool on, float) -> bf16x8 {
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (on) v = *reinterpret_cast<const u32x4*>(sV + i * kVStageStride + k);
                    return as_bf16x8(v);
                };
                expand_window_pipelined<NB>(acc[mb], my_slot, my_rank, my_scale, n_first, N, a.dv, sl.b_off, vfrag);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next window is staged
            }
        }

        if (m_ok) {
            if (FUSED) {
                uint16_t* orow = sl.out + (size_t)a.dv.perm[m] * N;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = n_first + nb * 32 + g * 8 + h * 4;
                        if (n < N) {
                            bf16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[mb][nb][g * 4 + e];
                            *reinterpret_cast<u32x2*>(orow + n) = __builtin_bit_cast(u32x2, o);
                        }
                    }
            } else {
                // fp32 partial tiles are kept block by block in accumulator order: block (m / 32, n / 32)
                // of split s is 1024 consecutive floats, lane (i, h) owning floats 256 g + 8 i + 4 h .. + 3,
                // so every store (and the matching load in the reduce kernel) covers 1 KB contiguously
                const int nblk_slice = (N + 31) / 32;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int bn = (n_first + nb * 32) / 32;          // block inside the slice
                    if (bn < nblk_slice) {
                        float* blk = a.part + (((size_t)split * (a.Mpad / 32) + (size_t)((m - a.m_begin) / 32)) * a.nblk + sl.blk0 + bn) * 1024;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            f32x4 o = {acc[mb][nb][g * 4 + 0], acc[mb][nb][g * 4 + 1], acc[mb][nb][g * 4 + 2],
                                       acc[mb][nb][g * 4 + 3]};
                            // read once by another kernel: keep the tiles from lingering dirty in L2
                            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(blk + g * 256 + i * 8 + h * 4));
                        }
                    }
                }
            }
        }
    }
}

}  // namespace lora
