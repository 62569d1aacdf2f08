// What a GEMM wavefront does with its finished accumulators; shared by the GEMM kernels.
//   fused path: LoRA expand on the accumulators (paper Sec. 2.2: the adapter's activations are added to the
//               backbone layer's output), one bf16 rounding, rows scattered back to token order;
//   split path: fp32 partial tile for the reduce + expand kernel.
//
// Accumulator layout ("W-first" orientation): acc[mb][nb] is a 32x32 block, lane (i, h) holds grouped row
// m_first + 32 mb + i and output columns n_first + 32 nb + 8 g + 4 h + e in register 4 g + e.
//
// The fused path works on the wave's windows (32 rows each) two at a time, in the wave's own piece of the LDS
// ring (free once every wave has left the main loop; the caller has synchronised):
//   1. the windows' scaled shrink results are parked there as bf16 and the expand runs as one pipelined pass
//      over the (window, slot) pairs;
//   2. the finished rows are rounded to bf16 and turned through the same piece of LDS, so that they leave as
//      16-byte stores in which consecutive lanes cover a whole run of an output row.  Written straight from the
//      accumulator layout, a store instruction touches 32 rows with 16 bytes each, and the output of a
//      256 x 256 tile reaches L2 as 8192 sixteen-byte pieces.
#pragma once

#include "device_common.hpp"

namespace lora {

constexpr int kEpiWindows = 2;                    // windows per pass
// expand work items in flight per wave: about 16 fragment loads (64 registers)
template <int NB>
constexpr int kExpandDepth = NB >= 4 ? 4 : (NB == 3 ? 5 : 8);
// bytes of the ring one wave uses in the fused epilogue: shrink results of two windows, or two windows of
// NB * 32 bf16 output columns
template <int NB>
constexpr int epilogue_bytes_per_wave()
{
    constexpr int v = kEpiWindows * kPieceRows * kVStageStride * 2, o = kEpiWindows * kPieceRows * NB * 64;
    return v > o ? v : o;
}

// Accumulators at the start of a tile: zero, or on the fused path the bias of the backbone layer where the
// projection has one (the q, k, v projections of the Qwen2.5 family): the products are then accumulated onto it
// in fp32 and it costs the epilogue neither loads nor registers.  The split path adds the bias once, in the
// reduce kernel.
template <int MB, int NB, bool FUSED>
__device__ __forceinline__ void init_accumulators(f32x16 (&acc)[MB][NB], const Slice& sl, int n_first)
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    if (!FUSED || sl.bias == nullptr) return;                     // uniform over the launch
    const int h = (threadIdx.x & (kWave - 1)) >> 5;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n_first + nb * 32 + g * 8 + h * 4;      // N is a multiple of 8: all four or none
            if (n < sl.N) {
                const bf16x4 b = __builtin_bit_cast(bf16x4, *reinterpret_cast<const u32x2*>(sl.bias + n));
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[mb][nb][g * 4 + e] = (float)b[e];
            }
        }
}

// Rounds WB windows of accumulators to bf16 and stores them to out rows perm[m], through LDS (sT: this wave's
// piece, WB * 32 rows of NB * 64 bytes).  Chunk c (16 bytes) of row r sits at position c ^ ((r >> 1) & (CH - 1))
// (CH a power of two; otherwise rotated by r >> 1): the 8-byte writes of a half wave then collide two ways at
// most and the 16-byte reads are contiguous.  One read instruction covers 64 / CH whole rows (with 12 chunks per
// row the last four lanes idle).
template <int WB, int NB>
__device__ __forceinline__ void store_windows(const f32x16 (&acc)[WB][NB], const GemmArgs& a, const Slice& sl, int m_first,
                                              int n_first, uint8_t* sT)
{
    constexpr int CH = NB * 4, ROWB = NB * 64;     // 16-byte chunks and bytes per LDS row
    constexpr bool P2 = (CH & (CH - 1)) == 0;
    constexpr int RPI = kWave / CH;                // rows one 16-byte-per-lane instruction covers
    constexpr int ROWS = WB * 32;
    constexpr int ITER = (ROWS + RPI - 1) / RPI;
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    const int T = a.m_end, N = sl.N;
    // row: inside its 32-row window
    auto place = [](int c, int row) { return P2 ? (c ^ ((row >> 1) & (CH - 1))) : (c + (row >> 1)) % CH; };
    auto chunk_at = [](int pos, int row) { return P2 ? (pos ^ ((row >> 1) & (CH - 1))) : (pos + CH - (row >> 1) % CH) % CH; };
    const int lrow = lane / CH, lpos = lane % CH;
    const bool lane_on = lrow < RPI;
    // tokens of the rows this lane will store (fetched before the LDS round trip)
    int tok[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int row = it * RPI + lrow;
        const int m = m_first + row;
        tok[it] = (lane_on && row < ROWS && m < T) ? a.dv.perm[m] : -1;
    }
#pragma unroll
    for (int w = 0; w < WB; ++w)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[w][nb][g * 4 + e];
                const int pos = place(nb * 4 + g, i);
                *reinterpret_cast<u32x2*>(sT + (w * 32 + i) * ROWB + pos * 16 + h * 8) = __builtin_bit_cast(u32x2, o);
            }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int row = it * RPI + lrow;
        if (tok[it] >= 0) {                                       // implies an existing row of this lane
            const int n = n_first + chunk_at(lpos, row & 31) * 8;
            const u32x4 v = *reinterpret_cast<const u32x4*>(sT + row * ROWB + lpos * 16);
            if (n < N) *reinterpret_cast<u32x4*>(sl.out + (size_t)tok[it] * N + n) = v;
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");            // reads done before the piece is reused
}

// Fused path, wave tiles of at most two 32-row windows: what the epilogue needs from memory besides the B rows
// is fetched ahead of it and waits in registers.  Two parts: what the segment map gives (slot and rank of the
// lane's rows; rank and scale of the rows whose shrink results the lane converts) is there before the launch and
// is fetched before the main loop; the shrink results themselves may come from workgroups of the same launch
// and are fetched once those have reported (prefetch_v), in one round of loads per K chunk.
template <int MB>
struct TilePrefetch {
    int slot[MB], rank[MB];          // this lane's row of each window
    int srank[MB][4];                // rank / scale of the row of each of this lane's four shares of a window
    float sscale[MB][4];
    f32x4 lo[MB][4], hi[MB][4];      // the shares as loaded (first K chunk), before scaling and rounding
    u32x4 v[MB][4];                  // this lane's shares of the windows' scaled shrink results (packed bf16)
};

template <int MB>
__device__ __forceinline__ void prefetch_rows(TilePrefetch<MB>& pf, const GemmArgs& a, int m_first)
{
    static_assert(MB <= kEpiWindows, "prefetch covers one pass");
    const int lane = threadIdx.x & (kWave - 1), i = lane & 31;
    const int last = a.m_end - 1;                                 // every load reads an existing row
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;
        const int mc = m < a.m_end ? m : last;
        const int s = a.dv.row_loc[mc], r = a.dv.row_rank[mc];
        pf.slot[mb] = m < a.m_end ? s : -1;
        pf.rank[mb] = m < a.m_end ? r : 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = lane + 64 * q;
            const int mr = m_first + mb * 32 + (idx >> 3);
            const bool on = mr < a.m_end && (idx & 7) * 8 < a.dv.max_rank;
            const int mrc = mr < a.m_end ? mr : last;
            const int rr = a.dv.row_rank[mrc];
            const float sc = a.dv.row_scale[mrc];
            pf.srank[mb][q] = on ? rr : 0;
            pf.sscale[mb][q] = on ? sc : 0.f;
            pf.v[mb][q] = u32x4{0u, 0u, 0u, 0u};
        }
    }
}

// Shares of the scaled shrink results: share q of window mb is (row, seg) = ((lane + 64 q) / 8, (lane + 64 q) % 8)
// -> bf16(scale_row * sum_c vpart[c][row][8 seg .. 8 seg + 7]), zero beyond the row's rank.  Every lane loads
// (lanes without a share read row 0 and drop the result), all shares of a K chunk in one round.  Two steps, so
// that the round trip of the first chunk can pass behind other work: prefetch_v_issue only requests it,
// prefetch_v_finish adds the other chunks (none when the shrink ran unsplit), scales and rounds.
template <int MB>
__device__ __forceinline__ const float* share_address(const TilePrefetch<MB>& pf, const GemmArgs& a, const Slice& sl,
                                                      int m_first, int mb, int q)
{
    const int idx = (threadIdx.x & (kWave - 1)) + 64 * q;
    const int mr = m_first + mb * 32 + (idx >> 3), seg = idx & 7;
    const bool live = seg * 8 < pf.srank[mb][q];               // implies the row exists
    return sl.vpart + (live ? (size_t)mr * a.dv.max_rank + seg * 8 : 0);
}

template <int MB>
__device__ __forceinline__ void prefetch_v_issue(TilePrefetch<MB>& pf, const GemmArgs& a, const Slice& sl, int m_first)
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float* vp = share_address(pf, a, sl, m_first, mb, q);
            pf.lo[mb][q] = *reinterpret_cast<const f32x4*>(vp);
            pf.hi[mb][q] = *reinterpret_cast<const f32x4*>(vp + 4);
        }
}

template <int MB>
__device__ __forceinline__ void prefetch_v_finish(TilePrefetch<MB>& pf, const GemmArgs& a, const Slice& sl, int m_first)
{
    const int lane = threadIdx.x & (kWave - 1);
    const size_t chunk = (size_t)a.dv.T * a.dv.max_rank;
    for (int c = 1; c < a.n_kc; ++c) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float* vp = share_address(pf, a, sl, m_first, mb, q) + c * chunk;
                pf.lo[mb][q] += *reinterpret_cast<const f32x4*>(vp);
                pf.hi[mb][q] += *reinterpret_cast<const f32x4*>(vp + 4);
            }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x8 vb;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vb[e] = (__bf16)(pf.lo[mb][q][e] * pf.sscale[mb][q]);
                vb[4 + e] = (__bf16)(pf.hi[mb][q][e] * pf.sscale[mb][q]);
            }
            const bool live = ((lane + 64 * q) & 7) * 8 < pf.srank[mb][q];
            pf.v[mb][q] = live ? __builtin_bit_cast(u32x4, vb) : u32x4{0u, 0u, 0u, 0u};
        }
}

// Epilogue of the fused path from prefetched window data.  ring: LDS free again (the caller has synchronised).
template <int MB, int NB>
__device__ __forceinline__ void finish_tile_prefetched(f32x16 (&acc)[MB][NB], const GemmArgs& a, const Slice& sl,
                                                       int m_first, int n_first, int wave, uint16_t* ring,
                                                       const TilePrefetch<MB>& pf)
{
    uint8_t* mine = reinterpret_cast<uint8_t*>(ring) + wave * epilogue_bytes_per_wave<NB>();
    bool any = false;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) any = any || __ballot(pf.slot[mb] >= 0 && pf.rank[mb] > 0) != 0;
    if (any) {                                                    // uniform over the wave
        uint16_t* sV = reinterpret_cast<uint16_t*>(mine);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q) park_v_share(sV + mb * kPieceRows * kVStageStride, q, pf.v[mb][q]);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        expand_windows<MB, NB, kExpandDepth<NB>>(acc, pf.slot, pf.rank, n_first, sl.N, a.dv, sl.b_unit, sV);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    store_windows<MB, NB>(acc, a, sl, m_first, n_first, mine);
}

// Fused path over a pair of projections of the same tokens whose product leaves the kernel (the gated MLP of the
// Llama and Qwen2.5 families, paper Sec. 8.1: h = silu(gate) * up is what `down` reads): acc[mb][2 j] holds columns
// n_first + 32 j .. of gate, acc[mb][2 j + 1] the same columns of up.  One window per pass: shrink results of both
// projections parked side by side, one expand pass over the window's slots with each block's own B and shrink
// results, then the activation and the product in fp32, one bf16 rounding, rows out through LDS.
constexpr int glu_epilogue_bytes_per_wave() { return 2 * kPieceRows * kVStageStride * 2; }

__device__ __forceinline__ float silu_f32(float z) { return z / (1.0f + __expf(-z)); }

template <int MB, int NB>
__device__ __forceinline__ void finish_tile_glu(f32x16 (&acc)[MB][NB], const GemmArgs& a, const Slice& gate, const Slice& up,
                                                int m_first, int n_first, int wave, uint16_t* ring)
{
    static_assert(NB % 2 == 0, "pairs of column blocks");
    static_assert(glu_epilogue_bytes_per_wave() >= kPieceRows * (NB / 2) * 64, "output rows fit the wave's piece");
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31;
    const int T = a.m_end, N = gate.N;
    uint8_t* mine = reinterpret_cast<uint8_t*>(ring) + wave * glu_epilogue_bytes_per_wave();
    uint16_t* sV = reinterpret_cast<uint16_t*>(mine);
    uint16_t* sV2 = sV + kPieceRows * kVStageStride;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;
        const bool ok = m < T;
        const int ps[1] = {ok ? a.dv.row_loc[m] : -1};
        const int pr[1] = {ok ? a.dv.row_rank[m] : 0};
        f32x16(&win)[1][NB] = *reinterpret_cast<f32x16(*)[1][NB]>(&acc[mb]);
        if (__ballot(ps[0] >= 0 && pr[0] > 0) != 0) {             // uniform over the wave
            u32x4 share[1][4], share2[1][4];
            window_v_shares<1>(share, gate.vpart, a.n_kc, m_first + mb * 32, a.dv);
            window_v_shares<1>(share2, up.vpart, a.n_kc, m_first + mb * 32, a.dv);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                park_v_share(sV, q, share[0][q]);
                park_v_share(sV2, q, share2[0][q]);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            expand_windows<1, NB, kExpandDepth<NB>, true>(win, ps, pr, n_first, N, a.dv, gate.b_unit, sV, up.b_unit, sV2);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the piece is reused
        }
        f32x16 prod[1][NB / 2];
#pragma unroll
        for (int j = 0; j < NB / 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) prod[0][j][v] = silu_f32(win[0][2 * j][v]) * win[0][2 * j + 1][v];
        store_windows<1, NB / 2>(prod, a, gate, m_first + mb * 32, n_first, mine);
    }
}

// ring: LDS no longer used by the main loop (the caller has synchronised).
template <int MB, int NB, bool FUSED>
__device__ __forceinline__ void finish_tile(f32x16 (&acc)[MB][NB], const GemmArgs& a, const Slice& sl, int m_first,
                                            int n_first, int split, int wave, uint16_t* ring)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    const int T = a.m_end, N = sl.N;
    if (FUSED) {
        // Windows two at a time: their rows' metadata and scaled shrink results are fetched together (one memory
        // latency each instead of one per window), then one pipelined pass over the (window, slot) pairs.
        constexpr int WB = MB >= kEpiWindows ? kEpiWindows : 1;
        static_assert(MB % WB == 0, "windows per wave");
        int slot[MB], rank[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = m_first + mb * 32 + i;
            const bool ok = m < T;
            slot[mb] = ok ? a.dv.row_loc[m] : -1;
            rank[mb] = ok ? a.dv.row_rank[m] : 0;
        }
        uint8_t* mine = reinterpret_cast<uint8_t*>(ring) + wave * epilogue_bytes_per_wave<NB>();
        uint16_t* sV = reinterpret_cast<uint16_t*>(mine);
#pragma unroll
        for (int p = 0; p < MB / WB; ++p) {
            f32x16(&pair)[WB][NB] = *reinterpret_cast<f32x16(*)[WB][NB]>(&acc[p * WB]);
            bool any = false;
#pragma unroll
            for (int w = 0; w < WB; ++w) any = any || __ballot(slot[p * WB + w] >= 0 && rank[p * WB + w] > 0) != 0;
            if (any) {                                            // uniform over the wave
                u32x4 share[WB][4];
                window_v_shares<WB>(share, sl.vpart, a.n_kc, m_first + p * WB * 32, a.dv);
#pragma unroll
                for (int w = 0; w < WB; ++w)
#pragma unroll
                    for (int q = 0; q < 4; ++q) park_v_share(sV + w * kPieceRows * kVStageStride, q, share[w][q]);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                int ps[WB], pr[WB];
#pragma unroll
                for (int w = 0; w < WB; ++w) {
                    ps[w] = slot[p * WB + w];
                    pr[w] = rank[p * WB + w];
                }
                expand_windows<WB, NB, kExpandDepth<NB>>(pair, ps, pr, n_first, N, a.dv, sl.b_unit, sV);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the piece is reused
            }
            store_windows<WB, NB>(pair, a, sl, m_first + p * WB * 32, n_first, mine);
        }
        return;
    }
    // split path: fp32 partial tiles are kept block by block in accumulator order: block (m / 32, n / 32) of
    // split s is 1024 consecutive floats, lane (i, h) owning floats 256 g + 8 i + 4 h .. + 3, so every store (and
    // the matching load in the reduce kernel) covers 1 KB contiguously
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m_first + mb * 32 + i;      // grouped row of this lane
        if (m >= T) continue;
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

}  // namespace lora
