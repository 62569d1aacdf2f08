// Base projection x W^T for large batches (prefill), where the matrix cores bound the kernel (paper Sec. 2.2: the
// adapter's activations are added to the backbone layer's output; Sec. 5.1.2: backbone latency grows linearly
// with the batch).
//
// Same tile as the other GEMM kernels - BM x BN per workgroup, MFMA 32x32x16 with W as first operand, K walked in
// 64-wide tiles of 128-byte rows, chunk c of row r at LDS position c ^ ((r >> 1) & 7) - but the tiles travel
// global -> registers -> LDS (ordinary loads, then ds_write) instead of through the global -> LDS copy
// instruction.  Measured on this chip, a CU fills its LDS through that instruction at 25 (four copying waves) to
// 43 (eight) bytes per clock from L2-resident data, and ordinary loads reach 56 - 60; a 256 x 256 tile at the full
// MFMA rate needs 64 KB per 2048 clocks = 32 bytes per clock, so the copy instruction, not the matrix cores, set
// the pace of the kernel that used it.  Registers also hold the tile in flight, so two LDS stages are enough:
// tile j is multiplied out of one stage while tile j + 1 (on its way since the first K step of tile j - 1) is written
// into the other during the first K step, and every register that write empties is refilled at once with its part of
// tile j + 2, which so has a whole tile time to arrive (refilling in the second K step left three quarters of one).
//
// One barrier per tile, in front of the MFMAs of the tile's last K step: every wave has its last fragments of
// tile j in registers by then (the stage may be overwritten) and has written its share of tile j + 1 (the
// stage may be read); the first fragments of tile j + 1 are requested right behind the barrier and the last K
// step's MFMAs cover their latency.
#include "gemm_epilogue.hpp"

#include <type_traits>
#include <utility>

namespace lora {
namespace {

template <typename F, int... Is>
__device__ __forceinline__ void staged_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void staged_for(F&& f)
{
    staged_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

constexpr int kSK = 64;        // K extent of one LDS tile (bf16 elements)
constexpr int kSRow = 128;     // bytes per LDS row

// LDS writes of this wave have landed, then meet the other waves.  No wait for global loads: the tile on its way
// into registers stays in flight across the barrier.
__device__ inline void lds_done_then_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// PG: tiles in flight in registers (1: compute-bound shapes, the tile's data comes from L2 within one tile time;
// 2: small batches, where the weight stream comes from HBM and bytes in flight set the rate).
// GLU: gate = slice 0 and up = slice 1 of the same tokens, silu(gate) * up stored; the W part of a stage alternates
// between the two matrices in blocks of 32 rows and a workgroup owns BN / 2 output columns (as in the 64-wide-K
// kernel for small batches).
template <int BM, int BN, int WGM, int WGN, int PG, bool GLU = false>
__global__ __launch_bounds__(WGM* WGN* kWave) void gemm_staged_kernel(GemmArgs a)
{
    constexpr int NWV = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;           // wave tile
    constexpr int MB = WTM / 32, NB = WTN / 32;             // 32x32 accumulator blocks per wave
    constexpr int STAGE_B = (BM + BN) * kSRow;              // bytes per stage
    constexpr int XQ = BM / 8 / NWV, WQ = BN / 8 / NWV;     // 16-byte loads per lane and tile (8 rows per wave load)
    static_assert(BM % (8 * NWV) == 0 && BN % (8 * NWV) == 0, "tile/waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    static_assert(2 * STAGE_B <= 160 * 1024, "LDS");
    static_assert(2 * STAGE_B >= NWV * epilogue_bytes_per_wave<NB>(), "ring too small for the fused epilogue");
    static_assert(!GLU || 2 * STAGE_B >= NWV * glu_epilogue_bytes_per_wave(), "ring too small for the gated epilogue");

    __shared__ __attribute__((aligned(1024))) uint8_t ring[2 * STAGE_B];

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave % WGM, wn = wave / WGM;
    const int T = a.m_end, K = a.K;                         // rows past m_end are computed, never stored

    // blockIdx -> (tile_m, tile_n): the M tile is the fastest index (neighbouring workgroups share the W tile)
    const int tile_m = (int)blockIdx.x % a.tiles_m, tile_n = (int)blockIdx.x / a.tiles_m;
    int si = 0;
    if (!GLU)
        for (int k = 1; k < a.g.n; ++k)
            if (tile_n >= a.g.s[k].tile0) si = k;
    const Slice sl = pick_slice(a.g, si);
    const int N = sl.N;
    // n0: first column inside the slice (GLU: first output column; the tile is BN / 2 of them wide)
    const int m0 = a.m_begin + tile_m * BM, n0 = (tile_n - sl.tile0) * (GLU ? BN / 2 : BN);
    const int nk = K / kSK;

    // Staging assignment: load q of wave w covers stage rows 8 (w XQ + q) .. + 7 of the x part (same for the W
    // part with WQ); lane l owns row l / 8 of those and its chunk l % 8, so eight lanes fetch one whole 128-byte
    // line.  Rows past T or N are clamped to the last valid row: they are computed, never stored.
    uint32_t xoff[XQ], woff[WQ];                            // byte offset of this lane's 16 bytes in tile 0
    uint32_t xst[XQ], wst[WQ];                              // byte offset of their place in a stage
    bool w_up[WQ];                                          // GLU: the rows of this load come from `up` (uniform over the wave)
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int r = (wave * XQ + q) * 8 + (lane >> 3), c = lane & 7;
        int m = m0 + r;
        if (m > T - 1) m = T - 1;
        xoff[q] = ((uint32_t)a.dv.perm[m] * (uint32_t)K + (uint32_t)(c * 8)) * 2u;
        xst[q] = (uint32_t)(r * kSRow + ((c ^ ((r >> 1) & 7)) << 4));
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int r = (wave * WQ + q) * 8 + (lane >> 3), c = lane & 7;
        int n = GLU ? n0 + (r >> 6) * 32 + (r & 31) : n0 + r;
        if (n > N - 1) n = N - 1;
        woff[q] = ((uint32_t)n * (uint32_t)K + (uint32_t)(c * 8)) * 2u;
        w_up[q] = GLU && ((((wave * WQ + q) * 8) >> 5) & 1);
        wst[q] = (uint32_t)((BM + r) * kSRow + ((c ^ ((r >> 1) & 7)) << 4));
    }
    const uint8_t* const xb = reinterpret_cast<const uint8_t*>(sl.x);
    const uint8_t* const wb = reinterpret_cast<const uint8_t*>(sl.W);
    const uint8_t* const wb_up = reinterpret_cast<const uint8_t*>(GLU ? a.g.s[1].W : sl.W);
    static_assert(PG == 1 || PG == 2, "register sets");
    u32x4 stg[PG][XQ + WQ];                                 // the tiles in flight: W parts first, then x parts
    constexpr int NST = XQ + WQ;
    auto load_one = [&](int set, int t, int q) {             // set, q: compile-time constants at every call site
        const size_t k0 = (size_t)t * (kSK * 2);
        stg[set][q] = q < WQ ? *reinterpret_cast<const u32x4*>((w_up[q] ? wb_up : wb) + k0 + woff[q])
                             : *reinterpret_cast<const u32x4*>(xb + k0 + xoff[q - WQ]);
    };
    auto store_one = [&](int set, int stage, int q) {
        uint8_t* st = ring + stage * STAGE_B;
        *reinterpret_cast<u32x4*>(st + (q < WQ ? wst[q] : xst[q - WQ])) = stg[set][q];
    };

    f32x16 acc[MB][NB];
    init_accumulators<MB, NB, !GLU>(acc, sl, n0 + wn * WTN);        // GLU: no bias (refused by the host)

    // byte offset of this lane's fragment of K step kk inside a 32-row block: row i, chunk 2 kk + h
    const int sw_i = (i >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) rd[kk] = i * kSRow + (((2 * kk + h) ^ sw_i) << 4);
    const int x_base = wm * WTM * kSRow, w_base = (BM + wn * WTN) * kSRow;

    bf16x8 Fw[2][NB], Fx[2][MB];
    constexpr int NM = MB * NB;                              // MFMAs per K step
    constexpr int NR = MB + NB;                              // LDS reads per K step
    static_assert(NR <= NM, "reads are spread one per MFMA");
    auto read_one = [&](int f, const uint8_t* st, int kk, int r) {      // f, kk, r: compile-time at every call site
        if (r < NB) Fw[f][r] = as_bf16x8(*reinterpret_cast<const u32x4*>(st + w_base + r * 32 * kSRow + rd[kk]));
        else Fx[f][r - NB] = as_bf16x8(*reinterpret_cast<const u32x4*>(st + x_base + (r - NB) * 32 * kSRow + rd[kk]));
    };
    auto mma_one = [&](int f, int t) {
        const int mb = t / NB, nb = t % NB;
        acc[mb][nb] = mfma32(Fw[f][nb], Fx[f][mb], acc[mb][nb]);
    };

    // prologue: tile 0 into stage 0, tiles 1 .. PG into the registers (tile t travels in register set t % PG)
    staged_for<NST>([&](auto q) { load_one(0, 0, q.value); });
    staged_for<NST>([&](auto q) { store_one(0, 0, q.value); });
    staged_for<PG>([&](auto d) {
        constexpr int t = decltype(d)::value + 1;
        if (t < nk) staged_for<NST>([&](auto q) { load_one(t % PG, t, q.value); });
    });
    lds_done_then_barrier();
    staged_for<NR>([&](auto r) { read_one(0, ring, 0, r.value); });

    // One tile.  STORE: tile j + 1 waits in its registers and goes into the other stage during K step 0; LOAD:
    // tile j + 1 + PG is requested into the same registers, each right behind the write that empties it; NEXT: there is a tile j + 1 to hand
    // over to.  SET: the register set of tile j + 1.  The instruction order is written out and pinned: behind
    // every MFMA one LDS read of the next K step's fragments and, in step 0, its share of the tile's LDS writes and
    // global loads, so that neither a row of writes that wait for their loads nor a row of reads stands
    // in front of the MFMAs (scheduling barriers: plain compiler fences do not hold MFMAs in place, they are not
    // memory operations).
    auto tile = [&](auto set_c, auto store_c, auto load_c, auto next_c, int j) {
        constexpr int SET = decltype(set_c)::value;
        constexpr bool STORE = decltype(store_c)::value, LOAD = decltype(load_c)::value, NEXT = decltype(next_c)::value;
        const uint8_t* st = ring + (j & 1) * STAGE_B;
        const int other = (j & 1) ^ 1;
        staged_for<NM>([&](auto tc) {                           // K step 0
            constexpr int t = decltype(tc)::value;
            mma_one(0, t);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (t < NR) read_one(1, st, 1, t);
            if constexpr (STORE)
                staged_for<(t + 1) * NST / NM - t * NST / NM>([&](auto q) {
                    store_one(SET, other, t * NST / NM + q.value);
                    if constexpr (LOAD) load_one(SET, j + 1 + PG, t * NST / NM + q.value);
                });
            __builtin_amdgcn_sched_barrier(0);
        });
        staged_for<NM>([&](auto tc) {                           // K step 1
            constexpr int t = decltype(tc)::value;
            mma_one(1, t);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (t < NR) read_one(0, st, 2, t);
            __builtin_amdgcn_sched_barrier(0);
        });
        staged_for<NM>([&](auto tc) {                           // K step 2
            constexpr int t = decltype(tc)::value;
            mma_one(0, t);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (t < NR) read_one(1, st, 3, t);
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (NEXT) lds_done_then_barrier();            // tile j + 1 is complete, tile j's stage is free
        staged_for<NM>([&](auto tc) {                           // K step 3
            constexpr int t = decltype(tc)::value;
            mma_one(1, t);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NEXT && t < NR) read_one(0, ring + other * STAGE_B, 0, t);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using Yes = std::true_type;
    using No = std::false_type;
    // tile j + 1 sits in register set (j + 1) % PG: with two sets the steady state walks two tiles per round so
    // that the set is a compile-time constant
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    if constexpr (PG == 1) {
        int j = 0;
        for (; j + 2 < nk; ++j) tile(S0{}, Yes{}, Yes{}, Yes{}, j);
        if (j + 1 < nk) {
            tile(S0{}, Yes{}, No{}, Yes{}, j);
            ++j;
        }
        if (j < nk) tile(S0{}, No{}, No{}, No{}, j);
    } else {
        int j = 0;                                               // even here and after every round
        for (; j + 4 < nk; j += 2) {                             // tiles j, j + 1: both store and load (j + 1 + 3 < nk)
            tile(S1{}, Yes{}, Yes{}, Yes{}, j);
            tile(S0{}, Yes{}, Yes{}, Yes{}, j + 1);
        }
        // at most four tiles are left, none of them loads except where a tile j + 3 still exists
        for (; j < nk; j += 2) {
            if (j + 3 < nk) tile(S1{}, Yes{}, Yes{}, Yes{}, j);
            else if (j + 1 < nk) tile(S1{}, Yes{}, No{}, Yes{}, j);
            else tile(S1{}, No{}, No{}, No{}, j);
            if (j + 1 < nk) {
                if (j + 2 < nk) tile(S0{}, Yes{}, No{}, Yes{}, j + 1);
                else tile(S0{}, No{}, No{}, No{}, j + 1);
            }
        }
    }

    // ---------------- epilogue ----------------
    __syncthreads();          // every wave has left the main loop: the ring is free
    if constexpr (GLU)
        finish_tile_glu<MB, NB>(acc, a, sl, a.g.s[1], m0 + wm * WTM, n0 + wn * (WTN / 2), wave, reinterpret_cast<uint16_t*>(ring));
    else
        finish_tile<MB, NB, true>(acc, a, sl, m0 + wm * WTM, n0 + wn * WTN, 0, wave, reinterpret_cast<uint16_t*>(ring));
}

template <int BM, int BN, int WGM, int WGN, int PG, bool GLU = false>
hipError_t launch_staged(GemmArgs a, hipStream_t stream)
{
    a.tiles_m = (a.m_end - a.m_begin + BM - 1) / BM;
    a.tiles_n = 0;
    if (GLU) {                                            // gate and up together: BN / 2 output columns per tile
        a.g.s[0].tile0 = a.g.s[1].tile0 = 0;
        a.tiles_n = (a.g.s[0].N + BN / 2 - 1) / (BN / 2);
    } else {
        for (int k = 0; k < a.g.n; ++k) {
            a.g.s[k].tile0 = a.tiles_n;
            a.tiles_n += (a.g.s[k].N + BN - 1) / BN;
        }
    }
    const int grid = a.tiles_m * a.tiles_n;
    hipLaunchKernelGGL((gemm_staged_kernel<BM, BN, WGM, WGN, PG, GLU>), dim3(grid), dim3(WGM * WGN * kWave), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_staged_glu(const GemmArgs& a, hipStream_t stream, const char** name)
{
    *name = "gemm_glu_staged_256x256x64_w8";
    return launch_staged<256, 256, 2, 4, 1, true>(a, stream);
}

hipError_t launch_gemm_staged_fused(const GemmArgs& a, int variant, hipStream_t stream, const char** name)
{
    switch (variant) {
        case 1:
            *name = "gemm_fused_staged_256x256x64_w4";
            return launch_staged<256, 256, 2, 2, 1>(a, stream);
        case 2:
            *name = "gemm_fused_staged_256x128x64_w8";
            return launch_staged<256, 128, 4, 2, 2>(a, stream);
        case 3:
            *name = "gemm_fused_staged_256x128x64_w8_pg1";
            return launch_staged<256, 128, 4, 2, 1>(a, stream);
        default:
            *name = "gemm_fused_staged_256x256x64_w8";
            return launch_staged<256, 256, 2, 4, 1>(a, stream);
    }
}

}  // namespace lora
