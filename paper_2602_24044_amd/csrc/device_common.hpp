// Device-side helpers shared by the HIP kernels: vector types, the MFMA 32x32x16 bf16 lane layout,
// the per-wavefront LoRA shrink work loop and the per-block LoRA expand.
#pragma once

#include "lora_internal.hpp"

namespace lora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline u32x4 load16(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] B[16x32].  Lane l = 32 h + i supplies A[i][8h..8h+7]
// and B[8h..8h+7][i]; it receives D[8 g + 4 h + e][i] in register 4 g + e (g, e in 0..3).
__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------------
// LoRA shrink, one work item per wavefront: item = (piece, K chunk).
//   vpart[kc][m][0:r] = sum_{k in chunk kc} x[perm[m], k] A_slot[j, k]        (paper Sec. 2.2)
// Operands come straight from global memory in MFMA layout.  Within a 64-wide K step lane (i, h)
// reads 64 contiguous bytes of row i at k0 + 32 h; MFMA q of the step consumes bytes [16 q, 16 q + 16)
// of both halves.  A and x use the same assignment, so the K order inside a step is permuted
// identically on both sides.  Several K steps are kept in flight (shrink_chunk).
// ---------------------------------------------------------------------------------------------------
struct ShrinkStep {
    u32x4 x[4], a0[4], a1[4];
};

// Every lane loads, also those whose row does not exist (their pointers are clamped to an existing row by the
// caller and what they produce is never stored): a predicated load is a branch, and behind branches the compiler
// can no longer count the loads in flight and waits for all of them before every step.
template <bool R64>
__device__ __forceinline__ void shrink_fetch(ShrinkStep& s, const uint16_t* xrow, const uint16_t* arow0, const uint16_t* arow1, int k0)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        s.x[q] = load16(xrow + k0 + q * 8);
        s.a0[q] = load16(arow0 + k0 + q * 8);
        if (R64) s.a1[q] = load16(arow1 + k0 + q * 8);
    }
}

template <bool R64>
__device__ __forceinline__ void shrink_mma(const ShrinkStep& s, f32x16& acc0, f32x16& acc1)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        acc0 = mfma32(as_bf16x8(s.a0[q]), as_bf16x8(s.x[q]), acc0);
        if (R64) acc1 = mfma32(as_bf16x8(s.a1[q]), as_bf16x8(s.x[q]), acc1);
    }
}

// K steps of one wavefront's share of an item, D of them in flight (each step is 8 or 12 independent 16-byte
// loads per lane; an item is a chain of dependent memory latencies, so the depth sets its duration).  The steady
// state is free of branches, so that the wait before a step covers that step's loads only.
template <bool R64>
__device__ __forceinline__ void shrink_chunk(const uint16_t* xrow, const uint16_t* arow0, const uint16_t* arow1, int k_begin,
                                    int k_end, f32x16& acc0, f32x16& acc1)
{
    constexpr int D = R64 ? 2 : 4;
    ShrinkStep st[D];
    int k0 = k_begin;
    if (k_end - k_begin >= 2 * D * kBK) {                    // uniform over the wave
#pragma unroll
        for (int d = 0; d < D; ++d) shrink_fetch<R64>(st[d], xrow, arow0, arow1, k0 + d * kBK);
        for (; k0 + 2 * D * kBK <= k_end; k0 += D * kBK) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                shrink_mma<R64>(st[d], acc0, acc1);
                shrink_fetch<R64>(st[d], xrow, arow0, arow1, k0 + (D + d) * kBK);
            }
        }
        // the D steps still in flight
#pragma unroll
        for (int d = 0; d < D; ++d) shrink_mma<R64>(st[d], acc0, acc1);
        k0 += D * kBK;
    }
    // what is left: fewer than 2 D steps, at most D at a time
    while (k0 < k_end) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (k0 + d * kBK < k_end) shrink_fetch<R64>(st[d], xrow, arow0, arow1, k0 + d * kBK);
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (k0 + d * kBK < k_end) shrink_mma<R64>(st[d], acc0, acc1);
        k0 += D * kBK;
    }
}

constexpr int kRedStride = 36;   // floats per LDS row of the cross-wave reduction (144 bytes: conflict-free)
constexpr int kRedFloatsPerWave = kPieceRows * kRedStride;

// Slice si of a packed group, picked with uniform selects over statically addressed kernel arguments (a
// dynamically indexed argument array would be fetched per lane and double the register count).
__device__ inline Slice pick_slice(const GroupArgs& g, int si)
{
    Slice r = g.s[0];
#pragma unroll
    for (int k = 1; k < kMaxGroup; ++k)
        if (si == k) r = g.s[k];
    return r;
}

// What the first work item of a workgroup needs before it can issue its operand loads; fetched at kernel
// start so that the chain item -> piece record -> perm -> x is off the critical path later.
struct ShrinkPrefetch {
    int n_items, n_pieces;
    int4 rec;      // piece record of the first item ({0, 0, -1, 0} when there is none)
    int tok;       // perm[rec.x + lane % 32]
};

// Work items are numbered (slice, piece, K chunk), the chunk fastest.
__device__ inline ShrinkPrefetch shrink_prefetch(const ShrinkArgs& a, int first_item)
{
    ShrinkPrefetch pf;
    const int i = threadIdx.x & 31;
    pf.n_pieces = *a.dv.n_pieces;
    pf.n_items = a.g.n * pf.n_pieces * a.n_kc;
    pf.rec = int4{0, 0, -1, 0};
    pf.tok = 0;
    if (first_item < pf.n_items) {
        pf.rec = reinterpret_cast<const int4*>(a.dv.piece_info)[(first_item / a.n_kc) % pf.n_pieces];
        if (i < pf.rec.y) pf.tok = a.dv.perm[pf.rec.x + i];
    }
    return pf;
}

// One shrink work item, processed by the whole workgroup of NW wavefronts: the waves split the item's K chunk
// between them, then the NW partial 32 x r blocks are summed through LDS (sRed: NW * kRedFloatsPerWave floats)
// and written as one partial result for the chunk.  rec / tok: the piece's record and this lane's token
// (perm[rec.x + lane % 32]).  Every branch on item data is uniform over the workgroup.
template <int NW>
__device__ inline void shrink_one_item(const ShrinkArgs& a, int item, int n_pieces, float* sRed, int4 rec, int tok)
{
    constexpr int NT = NW * kWave;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, h = lane >> 5;
    const int K = a.K;
    const int pk = item / a.n_kc;
    const int kc = item - pk * a.n_kc;
    const int si = pk / n_pieces;                       // slice (projection of a packed group)
    const Slice sl = pick_slice(a.g, si);
    const int m_begin = rec.x, nrows = rec.y, loc = rec.z, r = rec.w;
    if (loc < 0 || r <= 0) return;
    const int c_begin = kc * a.kc_len;
    int c_end = c_begin + a.kc_len;
    if (c_end > K) c_end = K;
    const int steps = (c_end - c_begin) / kBK;
    const int per_wave = (steps + NW - 1) / NW;
    const int k_begin = c_begin + wave * per_wave * kBK;
    int k_end = k_begin + per_wave * kBK;
    if (k_end > c_end) k_end = c_end;

    const uint16_t* xrow = sl.x + (size_t)tok * K + h * 32;
    const uint16_t* As = a.dv.slots + (size_t)loc * kLocUnit + (size_t)r * sl.a_unit;
    const bool a0_ok = i < r, a1_ok = (32 + i) < r;
    const uint16_t* arow0 = As + (size_t)(a0_ok ? i : 0) * K + h * 32;
    const uint16_t* arow1 = As + (size_t)(a1_ok ? 32 + i : 0) * K + h * 32;

    f32x16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;
    if (k_begin < k_end) {
        if (r <= 32) shrink_chunk<false>(xrow, arow0, arow1, k_begin, k_end, acc0, acc1);
        else shrink_chunk<true>(xrow, arow0, arow1, k_begin, k_end, acc0, acc1);
    }

    // accumulator: column = grouped row m_begin + i, register 4 g + e = rank index 8 g + 4 h + e
    const int halves = r > 32 ? 2 : 1;
    for (int half = 0; half < halves; ++half) {
        float* mine = sRed + wave * kRedFloatsPerWave + i * kRedStride;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = half ? acc1[g * 4 + e] : acc0[g * 4 + e];
            *reinterpret_cast<f32x4*>(mine + g * 8 + h * 4) = o;
        }
        __syncthreads();
        for (int idx = tid; idx < kPieceRows * 8; idx += NT) {
            const int row = idx >> 3, j4 = (idx & 7) * 4;
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < NW; ++w)
                sum += *reinterpret_cast<const f32x4*>(sRed + w * kRedFloatsPerWave + row * kRedStride + j4);
            const int j = half * 32 + j4;
            if (row < nrows && j < r)
                *reinterpret_cast<f32x4*>(sl.vpart + ((size_t)kc * a.dv.T + (size_t)(m_begin + row)) * a.dv.max_rank + j) = sum;
        }
        __syncthreads();
    }
}

// Processes work items first_item, first_item + stride, ... below end_item with the whole workgroup.  pf: the
// prefetched head of first_item.  An item starts with a chain of dependent loads (piece record -> token ->
// operands), each a full memory latency under the weight stream of the other workgroups; the chain is
// pipelined over three items: while item t is processed, the token of item t + 1 and the record of item t + 2
// are on their way.
template <int NW>
__device__ inline void shrink_block_items(const ShrinkArgs& a, int first_item, int stride, int end_item, float* sRed,
                                          const ShrinkPrefetch& pf)
{
    const int i = threadIdx.x & 31;
    const int n_pieces = pf.n_pieces;
    if (end_item > pf.n_items) end_item = pf.n_items;
    auto record = [&](int item) {
        int4 rec{0, 0, -1, 0};
        if (item < end_item) rec = reinterpret_cast<const int4*>(a.dv.piece_info)[(item / a.n_kc) % n_pieces];
        return rec;
    };
    auto token = [&](const int4& rec) { return (i < rec.y) ? a.dv.perm[rec.x + i] : 0; };
    int it0 = first_item, it1 = first_item + stride, it2 = first_item + 2 * stride;
    int4 r0 = pf.rec, r1 = record(it1);
    int t0 = pf.tok;
    while (it0 < end_item) {                                  // uniform over the workgroup
        const int4 r2 = record(it2);
        const int t1 = token(r1);
        shrink_one_item<NW>(a, it0, n_pieces, sRed, r0, t0);
        it0 = it1;
        it1 = it2;
        it2 += stride;
        r0 = r1;
        r1 = r2;
        t0 = t1;
    }
}

// This lane's share q (0 .. 3) of the scaled shrink results of one 32-row window, packed as bf16:
// (row, seg) = ((lane + 64 q) / 8, (lane + 64 q) % 8) -> bf16(scale_row * sum_c vpart[c][row][8 seg .. 8 seg + 7]),
// zero beyond the row's rank.
constexpr int kVStageStride = kMaxRank + 8;     // 144-byte rows: conflict-free 16-byte reads
__device__ inline u32x4 window_v_share(int q, const float* vpart, int n_kc, int win0, const DeviceView& dv)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int T = dv.T;
    const int idx = lane + 64 * q;
    const int row = idx >> 3, seg = idx & 7;
    const int mr = win0 + row;
    u32x4 packed = {0u, 0u, 0u, 0u};
    if (mr < T && seg * 8 < dv.max_rank) {
        const int r = dv.row_rank[mr];
        const float sc = dv.row_scale[mr];
        if (seg * 8 < r) {
            f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
            for (int c = 0; c < n_kc; ++c) {
                const float* vp = vpart + ((size_t)c * T + mr) * dv.max_rank + seg * 8;
                lo += *reinterpret_cast<const f32x4*>(vp);
                hi += *reinterpret_cast<const f32x4*>(vp + 4);
            }
            bf16x8 vb;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vb[e] = (__bf16)(lo[e] * sc);
                vb[4 + e] = (__bf16)(hi[e] * sc);
            }
            packed = __builtin_bit_cast(u32x4, vb);
        }
    }
    return packed;
}

// The four shares of each of WB consecutive windows.  One share after the other would be a chain of 4 * n_kc
// dependent memory latencies per window (every chunk's partial is added before the next is requested); here the
// row data of all windows is requested together, then per window and chunk the partials of its four shares in
// one go: 1 + WB * n_kc latencies.  The partials are loaded by every lane (a predicated load is a branch that
// keeps the compiler from overlapping the loads); lanes without a share read row 0 and drop the result.
template <int WB>
__device__ __forceinline__ void window_v_shares(u32x4 (&share)[WB][4], const float* vpart, int n_kc, int win0,
                                                const DeviceView& dv)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int T = dv.T;
    int r[WB][4];
    float sc[WB][4];
#pragma unroll
    for (int w = 0; w < WB; ++w)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = lane + 64 * q;
            const int mr = win0 + w * kPieceRows + (idx >> 3);
            const bool on = mr < T && (idx & 7) * 8 < dv.max_rank;
            r[w][q] = on ? dv.row_rank[mr] : 0;
            sc[w][q] = on ? dv.row_scale[mr] : 0.f;
        }
    const size_t chunk = (size_t)T * dv.max_rank;
#pragma unroll
    for (int w = 0; w < WB; ++w) {
        const float* vp[4];
        f32x4 lo[4], hi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = lane + 64 * q;
            const int mr = win0 + w * kPieceRows + (idx >> 3), seg = idx & 7;
            const bool live = seg * 8 < r[w][q];              // implies the row exists
            vp[q] = vpart + (live ? (size_t)mr * dv.max_rank + seg * 8 : 0);
            lo[q] = hi[q] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int c = 0; c < n_kc; ++c) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo[q] += *reinterpret_cast<const f32x4*>(vp[q] + c * chunk);
                hi[q] += *reinterpret_cast<const f32x4*>(vp[q] + c * chunk + 4);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bf16x8 vb;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vb[e] = (__bf16)(lo[q][e] * sc[w][q]);
                vb[4 + e] = (__bf16)(hi[q][e] * sc[w][q]);
            }
            const bool live = ((lane + 64 * q) & 7) * 8 < r[w][q];
            share[w][q] = live ? __builtin_bit_cast(u32x4, vb) : u32x4{0u, 0u, 0u, 0u};
        }
    }
}

// Parks share q in the window's LDS image (sV: 32 rows of kVStageStride elements).
__device__ inline void park_v_share(uint16_t* sV, int q, u32x4 packed)
{
    const int idx = (threadIdx.x & (kWave - 1)) + 64 * q;
    *reinterpret_cast<u32x4*>(sV + (idx >> 3) * kVStageStride + (idx & 7) * 8) = packed;
}

// ---------------------------------------------------------------------------------------------------
// LoRA expand for MB consecutive 32-row windows held by one wavefront, as one pipelined pass over work items
// (window, distinct slot, K step of 16 ranks): an adapter of rank 8 or 16 is one item per window it appears in,
// rank 32 two, rank 64 four.  Every item is NB loads of 16 bytes per lane (the B fragments of its rank range, one
// per 32-column block) and NB MFMAs; the fragments of the next D - 1 items are in flight while the current
// item's MFMAs run, across pair and window boundaries (the fragments are a dependent global load: the depth of
// the ring sets the duration of the pass).  The loads are unconditional and the same number for every item, also
// for the D - 1 items requested past the end of the list (they read the start of the slot region): loads behind
// a branch, or a number of loads that depends on the adapter, would leave the compiler unable to tell an item's
// own loads from the younger ones, and every item would wait for all loads in flight.  Lanes whose column or
// rank range does not exist read an existing place (row N - 1, rank offset 0); what they load is replaced by zeros.
// slot / rank: the lane's row of each window; `slot` holds the location of the row's adapter in the slot region
// (DeviceView::row_loc: one value per resident adapter, so it also tells adapters apart; -1 or rank 0: backbone only).  sV: the windows' scaled
// shrink results in LDS, window mb at sV + mb * kPieceRows * kVStageStride.
// ---------------------------------------------------------------------------------------------------
// GLU: the column blocks alternate between two projections of the same tokens (block 2 j: columns n_first + 32 j ..
// of the first, block 2 j + 1: the same columns of the second), each with its own B (b_unit / b_unit2) and its own
// shrink results (sV / sV2).
template <int MB, int NB, int D, bool GLU = false>
__device__ inline void expand_windows(f32x16 (&acc)[MB][NB], const int (&slot)[MB], const int (&rank)[MB], int n_first,
                                      int N, const DeviceView& dv, size_t b_unit, const uint16_t* sV, size_t b_unit2 = 0,
                                      const uint16_t* sV2 = nullptr)
{
    static_assert(!GLU || NB % 2 == 0, "pairs of column blocks");
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & 31, h = lane >> 5;
    unsigned long long todo[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) todo[mb] = __ballot(slot[mb] >= 0 && rank[mb] > 0);
    struct Item {
        int mb, s, r, ks;
        bool valid;
    };
    Item cur{0, 0, 8, 0, false};                              // the pair the generator is inside of
    auto next_item = [&]() {
        if (cur.valid && (cur.ks + 1) * 16 < cur.r) {         // uniform over the wave
            ++cur.ks;
            return cur;
        }
        Item q{0, 0, 8, 0, false};
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (!q.valid && todo[mb]) {                       // uniform over the wave
                const int leader = __ffsll((long long)todo[mb]) - 1;
                q.mb = mb;
                q.s = __builtin_amdgcn_readfirstlane(__shfl(slot[mb], leader, kWave));
                q.r = __builtin_amdgcn_readfirstlane(__shfl(rank[mb], leader, kWave));
                q.valid = true;
                todo[mb] &= ~__ballot(slot[mb] == q.s);
            }
        }
        cur = q;
        return q;
    };
    struct Frag {
        u32x4 f[NB];
    };
    // an item past the end of the list has s = 0, r = 8, ks = 0: the first bytes of the slot region
    auto fetch = [&](const Item& q, Frag& fb) {
        const int k = q.ks * 16 + h * 8;
        const int kc = k < q.r ? k : 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            int n = n_first + (GLU ? (nb >> 1) : nb) * 32 + i;
            if (n > N - 1) n = N - 1;
            const size_t bu = (GLU && (nb & 1)) ? b_unit2 : b_unit;
            const uint16_t* Bs = dv.slots + (size_t)q.s * kLocUnit + ((size_t)q.r * bu + (size_t)n * q.r);
            fb.f[nb] = load16(Bs + kc);
        }
    };
    auto apply = [&](const Item& q, const Frag& fb) {
        int my = slot[0];
#pragma unroll
        for (int mb = 1; mb < MB; ++mb)
            if (q.mb == mb) my = slot[mb];
        const int k = q.ks * 16 + h * 8;
        const bool k_on = k < q.r;                            // beyond the rank the lane loaded a stand-in
        const uint16_t* vrow = sV + (q.mb * kPieceRows + i) * kVStageStride;
        u32x4 v = {0u, 0u, 0u, 0u}, v2 = {0u, 0u, 0u, 0u};
        if (my == q.s && k_on) {
            v = *reinterpret_cast<const u32x4*>(vrow + k);
            if (GLU) v2 = *reinterpret_cast<const u32x4*>(sV2 + (q.mb * kPieceRows + i) * kVStageStride + k);
        }
        const bf16x8 vf = as_bf16x8(v), vf2 = as_bf16x8(v2);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (q.mb == mb) {                                 // uniform over the wave
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const u32x4 bf = k_on ? fb.f[nb] : u32x4{0u, 0u, 0u, 0u};
                    acc[mb][nb] = mfma32(as_bf16x8(bf), (GLU && (nb & 1)) ? vf2 : vf, acc[mb][nb]);
                }
            }
        }
    };
    // ring of D items, consumed in ring order; position d is refilled right after its item has been applied
    Frag f[D];
    Item q[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        q[d] = next_item();
        fetch(q[d], f[d]);
    }
    while (q[0].valid) {                                      // a pass without an item at position 0 has none at all
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (q[d].valid) apply(q[d], f[d]);                // uniform over the wave
            q[d] = next_item();
            fetch(q[d], f[d]);
        }
    }
}

}  // namespace lora
