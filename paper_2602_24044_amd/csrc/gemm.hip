// Base projection x W^T on the bf16 matrix cores (paper Sec. 2.2: the adapter's activations are added
// to the backbone layer's output; Sec. 1: the backbone is shared, adapters stay unmerged).
//
// Rows of the GEMM are grouped positions m (token perm[m]); x rows are gathered through perm when the
// tile is staged and output rows are scattered back through it, so `out` is in token order.
//
// Tiling: BM x BN output tile per workgroup, K walked in 32-wide tiles through a ring of NS LDS stages.
// Tiles are copied global -> LDS directly (global_load_lds, 16 bytes per lane: no staging registers, no
// LDS store instructions); one wave instruction fills 1 KB = 16 LDS rows of 64 bytes.  A stage holds the
// BM x-rows followed by the BN W-rows.  Chunk c (16 bytes) of row rr sits at position c ^ ((rr >> 2) & 3);
// because the copy engine places lane l at byte 16 l of the wave's 1 KB, the swizzle is applied on the
// global side (lane l fetches the chunk that belongs at its position).  The LDS serves a 128-bit read 16
// lanes per cycle over 64 banks, the 16 lanes being those of a 32-lane half whose lane-index bits 2, 3, 4
// have equal parity; with this swizzle the 16 rows of such a group fall on 16 different 16-byte bank
// groups, so the MFMA-layout reads (32 rows x one chunk) are bank-conflict free.  NS - 2 tile copies stay in flight behind the tile being
// multiplied, which is what covers the HBM latency (see the main loop for the schedule).
//
// MFMA 32x32x16 bf16 with W as the first operand and x as the second: the accumulator of a lane then
// holds one grouped row m (its column index) and, per group of four registers, four consecutive
// output columns n, so results leave as 8-byte (bf16) or 16-byte (fp32) stores.
//
// FUSED: K is walked in full; the LoRA expand runs on the accumulators (expand_window) and the result
//        is rounded once to bf16.
// SPLITK: blockIdx selects a K range; fp32 partial tiles go to the reduce + expand kernel.  After its
//        tile, every workgroup takes a share of the LoRA shrink work items of the same projection, so
//        shrink and base GEMM share one launch.
#include "gemm_epilogue.hpp"

#include <type_traits>
#include <utility>

namespace lora {
namespace {

constexpr int kTK = 32;   // K extent of one LDS tile (bf16 elements): 64-byte rows

template <typename F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ inline void static_for(F&& f)
{
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// One global -> LDS copy instruction: every lane hands in the address of its 16 bytes, the wave's 1 KB
// lands at lds_addr (wave-uniform) + 16 * lane.  Issued from inline assembly so that the only ordering
// against later LDS reads is the explicit vmcnt wait + barrier of the main loop (the compiler would
// otherwise drain all copies before any LDS read whose stage it cannot tell apart).
__device__ inline void copy16_to_lds(const void* base, uint32_t byte_off, uint32_t lds_addr)
{
    // base: wave-uniform address (a scalar register pair), byte_off: this lane's offset from it.  The address of a
    // tile then advances with scalar additions and the copy needs no vector ALU instruction at all: in the
    // compute-bound kernels those share the issue port with the MFMAs.
    // m0 carries the LDS address.  It cannot be named as a clobber (a reserved register: the compiler rejects
    // it) and needs none: the compiler keeps no value in m0 between statements, it writes m0 itself directly in
    // front of each instruction of its own that reads it.  Putting the old value back after the copy was tried
    // and stalls every copy (the write to m0 waits until the copy instruction has read it): + 0.2 us per K tile.
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory");
}

template <int N>
__device__ inline void wait_copies_then_barrier()
{
    // at most N of this wave's tile-copy instructions may still be in flight; then meet the other waves
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// ALLCOPY (fused path only): every wave copies, as on the split path: right for small batches, where the copy
// rate and not the MFMA issue bounds the loop.
template <int BM, int BN, int WGM, int WGN, bool FUSED, int NS, bool ALLCOPY = false>
__global__ __launch_bounds__(WGM* WGN* kWave) void gemm_kernel(GemmArgs a, ShrinkArgs sa)
{
    constexpr int NWV = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;           // wave tile
    constexpr int MB = WTM / 32, NB = WTN / 32;             // 32x32 accumulator blocks per wave
    constexpr int STAGE = (BM + BN) * kTK;                  // elements per stage
    // On the fused path only the first CW waves (one per SIMD) issue tile copies.  A wave that is held at a
    // copy instruction by a full memory pipeline cannot issue its MFMAs; with two waves per SIMD the other
    // one keeps the matrix core busy meanwhile (measured: a few percent on the compute-bound shapes, none
    // on the split path, where every wave copies).
    constexpr int CW = (FUSED && NWV > 4 && !ALLCOPY) ? 4 : NWV;
    constexpr int XQ = BM / 16 / CW, WQ = BN / 16 / CW;     // copy instructions per copying wave and tile
    constexpr int QPT = XQ + WQ;
    static_assert(BM % (16 * CW) == 0 && BN % (16 * CW) == 0, "tile/waves");
    static_assert(NS >= 3 && NS <= 8, "stages");
    static_assert((NS - 2) * QPT <= 63, "vmcnt range");

    // ring of NS stages; the copy instructions address it by LDS byte address, the MFMA loop reads it
    __shared__ __attribute__((aligned(1024))) uint16_t ring[NS * STAGE];
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)ring;

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);    // a scalar: what depends on it alone stays scalar
    const int i = lane & 31, h = lane >> 5;
    const int cwave = wave;                                 // index among the copying waves
    const int wm = wave % WGM, wn = (wave / WGM) % WGN;
    const int T = a.m_end, K = a.K;                         // rows past m_end are computed, never stored

    // blockIdx -> (split, tile_m, tile_n).  Consecutive blockIdx values land on different XCDs, so
    // the K split is the fastest index on the split path (every XCD keeps one x K-range in its L2)
    // and the M tile is the fastest on the fused path (neighbouring workgroups share the W tile).
    int split = 0, tile_m, tile_n;
    {
        int b = blockIdx.x;
        if (!FUSED) {
            split = b % a.split_k;
            b /= a.split_k;
        }
        tile_m = b % a.tiles_m;
        tile_n = b / a.tiles_m;
    }
    // the slice (projection of a packed group) this N tile belongs to; uniform over the workgroup
    int si = 0;
    for (int k = 1; k < a.g.n; ++k)
        if (tile_n >= a.g.s[k].tile0) si = k;
    const Slice sl = pick_slice(a.g, si);
    const uint16_t* const xg = sl.x;
    const uint16_t* const Wg = sl.W;
    const int N = sl.N;
    const int m0 = a.m_begin + tile_m * BM, n0 = (tile_n - sl.tile0) * BN;      // n0: column inside the slice

    // split path: metadata of this workgroup's first shrink work item, fetched before the main loop
    ShrinkPrefetch spf{};
    if (!FUSED && sa.on) spf = shrink_prefetch(sa, blockIdx.x);

    const int kt_total = K / kTK;
    int kt_begin = 0, kt_end = kt_total;
    if (!FUSED) {
        kt_begin = (int)((long long)kt_total * split / a.split_k);
        kt_end = (int)((long long)kt_total * (split + 1) / a.split_k);
    }
    const int nk = kt_end - kt_begin;

    // Copy assignment: copy instruction q of wave w fills stage rows 16 (w XQ + q) .. + 15 (x part; same
    // for the W part with WQ); lane l owns row l / 4 of those and chunk position l % 4.  Rows past T or N
    // are clamped to the last valid row: they are computed, never stored.
    const int cp_row = lane >> 2;
    const int cp_chunk = (lane & 3) ^ ((cp_row >> 2) & 3);
    uint32_t xoff[XQ], woff[WQ];                            // byte offsets of this lane's 16 bytes in tile 0
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        int m = m0 + (cwave * XQ + q) * 16 + cp_row;
        if (m > T - 1) m = T - 1;
        xoff[q] = ((uint32_t)a.dv.perm[m] * (uint32_t)K + (uint32_t)(cp_chunk * 8 + kt_begin * kTK)) * 2u;
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        int n = n0 + (cwave * WQ + q) * 16 + cp_row;
        if (n > N - 1) n = N - 1;
        woff[q] = ((uint32_t)n * (uint32_t)K + (uint32_t)(cp_chunk * 8 + kt_begin * kTK)) * 2u;
    }

    f32x16 acc[MB][NB];
    init_accumulators<MB, NB, FUSED>(acc, sl, n0 + wn * WTN);

    // ---- software-pipelined main loop ----
    // Tile j lives in stage j % NS.  State at the top of iteration j: tile j has landed for every wave,
    // the fragments of its first K step are in F[0], and the copies of tiles j + 1 .. j + NS - 2 are in
    // flight or landed.  K step 0 runs its MFMAs with the LDS reads of step 1 spread between them.  The
    // wave then waits until its own share of tile j + 1 has landed (younger copies stay in flight) and
    // meets the other waves at the barrier: tile j + 1 is now complete for everyone and the stage of tile
    // j - 1 is free.  K step 1 runs its MFMAs with the copy instructions of tile j + NS - 1 (into the freed
    // stage) and the LDS reads of tile j + 1's first fragments spread between them, so neither the copy
    // issue nor the LDS latency ever leaves the matrix core idle.  Instruction order is pinned with
    // scheduling barriers; without them the compiler batches all MFMAs of a step together.
    bf16x8 Fw[2][NB], Fx[2][MB];
    const int sw = (i >> 2) & 3;                              // (row >> 2) & 3 of every row this lane reads
    constexpr int NM = MB * NB;                               // MFMAs per K step
    constexpr int NR = MB + NB;                               // LDS reads per K step
    const uint32_t cp_x = ring_addr + cwave * XQ * 1024;      // this wave's first x / W copy target in stage 0
    const uint32_t cp_w = ring_addr + BM * kTK * 2 + cwave * WQ * 1024;
    const int rd_lane[2] = {i * kTK + ((0 * 2 + h) ^ sw) * 8, i * kTK + ((1 * 2 + h) ^ sw) * 8};

    const bool copier = wave < CW;
    auto copy_one = [&](int stage, int q, uint32_t k0) {      // q: compile-time constant at every call site
        if (!copier) return;
        const uint32_t so = (uint32_t)stage * (STAGE * 2);
        if (q < XQ)
            copy16_to_lds(xg + k0, xoff[q], cp_x + so + q * 1024);
        else
            copy16_to_lds(Wg + k0, woff[q - XQ], cp_w + so + (q - XQ) * 1024);
    };
    auto read_one = [&](auto f_c, int stage, int kk, int r) { // kk, r: compile-time constants at every call site
        constexpr int Fi = decltype(f_c)::value;
        const uint16_t* base = ring + stage * STAGE + rd_lane[kk];
        if (r < NB)
            Fw[Fi][r] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + (BM + wn * WTN + r * 32) * kTK));
        else
            Fx[Fi][r - NB] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + (wm * WTM + (r - NB) * 32) * kTK));
    };
    auto mma_one = [&](auto f_c, int t) {                     // t: compile-time constant at every call site
        constexpr int Fi = decltype(f_c)::value;
        const int mb = t / NB, nb = t % NB;
        acc[mb][nb] = mfma32(Fw[Fi][nb], Fx[Fi][mb], acc[mb][nb]);
    };
    // young = number of younger tile copies that may stay in flight behind the one being waited for
    auto wait_barrier = [&](int young) {
        // waiting with a smaller allowance than necessary is always safe
        if (NS > 7 && young >= 6) wait_copies_then_barrier<(NS > 7 ? 6 : 0) * QPT>();
        else if (NS > 6 && young >= 5) wait_copies_then_barrier<(NS > 6 ? 5 : 0) * QPT>();
        else if (NS > 5 && young >= 4) wait_copies_then_barrier<(NS > 5 ? 4 : 0) * QPT>();
        else if (NS > 4 && young >= 3) wait_copies_then_barrier<(NS > 4 ? 3 : 0) * QPT>();
        else if (NS > 3 && young >= 2) wait_copies_then_barrier<(NS > 3 ? 2 : 0) * QPT>();
        else if (young >= 1) wait_copies_then_barrier<1 * QPT>();
        else wait_copies_then_barrier<0>();
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // cur / nxt: stages of tiles j and j + 1.  fre0: stage of tile j - 2, freed at the previous barrier; it
    // receives the second half of tile j + NS - 2's copy during K step 0.  fre1: stage of tile j - 1, freed
    // at this iteration's barrier; it receives the first half of tile j + NS - 1's copy during K step 1.
    // Splitting each tile copy over two K steps keeps the copy issue rate even, so a wave is rarely held
    // up behind a full memory pipeline with MFMAs waiting behind it.
    constexpr int QA = (QPT + 1) / 2, QB = QPT - QA;          // first / second half of a tile copy
    auto iteration = [&](auto copy_c, int j, int cur, int nxt, int fre0, int fre1) {
        constexpr bool COPY = decltype(copy_c)::value;
        // K step 0: MFMAs on F[0]; second half of the copy of tile j + NS - 2; reads of step 1 into F[1]
        {
            const uint32_t k0 = (uint32_t)(j + NS - 2) * kTK;
            constexpr int NI = (COPY ? QB : 0) + NR;
            static_for<NM>([&](auto t) {
                mma_one(I0{}, t.value);
                asm volatile("" ::: "memory");
                static_for<NI>([&](auto it) {
                    if constexpr (it.value * NM / NI == t.value) {
                        if constexpr (COPY && it.value >= NR) copy_one(fre0, QA + it.value - NR, k0);
                        else read_one(I1{}, cur, 1, it.value);
                    }
                });
                asm volatile("" ::: "memory");
            });
        }
        // own share of tile j + 1 landed (younger copy instructions may stay in flight), then barrier
        if constexpr (COPY) {
            wait_copies_then_barrier<(NS - 3) * QPT>();
        } else {
            int young = nk - 2 - j;           // complete tile copies issued after tile j + 1
            if (young < 0) young = 0;
            if (young > NS - 3) young = NS - 3;
            wait_barrier(young);
        }
        // K step 1: MFMAs on F[1]; first half of the copy of tile j + NS - 1; reads of tile j + 1, step 0
        {
            const uint32_t k0 = (uint32_t)(j + NS - 1) * kTK;
            constexpr int NI = (COPY ? QA : 0) + NR;
            static_for<NM>([&](auto t) {
                mma_one(I1{}, t.value);
                asm volatile("" ::: "memory");
                static_for<NI>([&](auto it) {
                    if constexpr (it.value * NM / NI == t.value) {
                        // the reads first: the next iteration's first MFMA needs all of them
                        if constexpr (it.value < NR) read_one(I0{}, nxt, 0, it.value);
                        else copy_one(fre1, it.value - NR, k0);
                    }
                });
                asm volatile("" ::: "memory");
            });
        }
    };

    {
        // Prologue: tiles 0 .. NS - 3 in full and the first half of tile NS - 2 (its second half follows in
        // K step 0 of iteration 0, exactly as in the steady state).
        const bool steady = nk >= NS;              // at least one steady-state iteration exists
        if (nk > 0) {
            static_for<NS - 2>([&](auto d) {
                if (d.value < nk) {
                    static_for<QPT>([&](auto q) { copy_one(d.value, q.value, (uint32_t)d.value * kTK); });
                }
            });
            if (NS - 2 < nk) {
                if (steady) {
                    static_for<QA>([&](auto q) { copy_one(NS - 2, q.value, (uint32_t)(NS - 2) * kTK); });
                } else {
                    static_for<QPT>([&](auto q) { copy_one(NS - 2, q.value, (uint32_t)(NS - 2) * kTK); });
                }
            }
            // wait for tile 0: everything younger may stay in flight
            int young_instr = 0;
            {
                const int full = (nk - 1 < NS - 3) ? nk - 1 : NS - 3;      // complete younger tiles among 1 .. NS - 3
                young_instr = (full > 0 ? full : 0) * QPT;
                if (NS - 2 < nk && NS - 2 >= 1) young_instr += steady ? QA : QPT;
            }
            // round the allowance down to a multiple the wait helper knows (waiting for more is always safe)
            wait_barrier(young_instr / QPT > NS - 2 ? NS - 2 : young_instr / QPT);
            static_for<NR>([&](auto r) { read_one(I0{}, 0, 0, r.value); });
        }
        {
            int cur = 0, nxt = 1 % NS, fre1 = NS - 1, fre0 = NS - 2;
            int j = 0;
            auto advance = [&]() {
                fre0 = fre1;
                fre1 = cur;
                cur = nxt;
                nxt = (nxt + 1 == NS) ? 0 : nxt + 1;
            };
            if (steady) {
                for (; j + NS - 1 < nk; ++j) {    // steady state: one tile copy issued per iteration
                    iteration(std::true_type{}, j, cur, nxt, fre0, fre1);
                    advance();
                }
                // the first half of tile nk - 1 is out; send its second half before draining
                static_for<QB>([&](auto q) { copy_one(fre0, QA + q.value, (uint32_t)(nk - 1) * kTK); });
            }
            for (; j < nk; ++j) {                 // drain: the remaining tiles are already on their way
                iteration(std::false_type{}, j, cur, nxt, fre0, fre1);
                advance();
            }
        }

    }

    // ---------------- epilogue ----------------
    // every copy has landed and been read once all waves have left the main loop: the ring is free
    static_assert(!FUSED || NS * STAGE * 2 >= NWV * epilogue_bytes_per_wave<NB>(), "ring too small for the fused epilogue");
    static_assert(FUSED || NS * STAGE * 2 >= NWV * kRedFloatsPerWave * 4, "ring too small for the reduction");
    if (FUSED) __syncthreads();
    finish_tile<MB, NB, FUSED>(acc, a, sl, m0 + wm * WTM, n0 + wn * WTN, split, wave, ring);
    if (!FUSED && sa.on) {
        __syncthreads();
        shrink_block_items<NWV>(sa, blockIdx.x, gridDim.x, spf.n_items, reinterpret_cast<float*>(ring), spf);
    }
}

template <int BM, int BN, int WGM, int WGN, bool FUSED, int NS, bool ALLCOPY = false>
hipError_t launch_one(const GemmArgs& a, const ShrinkArgs& sa, hipStream_t stream)
{
    constexpr int NT = WGM * WGN * kWave;
    auto kfn = gemm_kernel<BM, BN, WGM, WGN, FUSED, NS, ALLCOPY>;
    const int grid = a.tiles_m * a.tiles_n * (FUSED ? 1 : a.split_k);
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), 0, stream, a, sa);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_fused(const GemmArgs& a0, int variant, hipStream_t stream, const char** name)
{
    GemmArgs a = a0;
    ShrinkArgs none{};
    none.on = 0;
    auto tiles = [&](int BM, int BN) {
        a.tiles_m = (a.m_end - a.m_begin + BM - 1) / BM;
        a.tiles_n = 0;
        for (int k = 0; k < a.g.n; ++k) {
            a.g.s[k].tile0 = a.tiles_n;
            a.tiles_n += (a.g.s[k].N + BN - 1) / BN;
        }
    };
    switch (variant) {
        case 1:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w4";
            return launch_one<256, 256, 2, 2, true, 4>(a, none, stream);
        case 2:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w4_s3";
            return launch_one<256, 256, 2, 2, true, 3>(a, none, stream);
        case 3:
            tiles(128, 128);
            *name = "gemm_fused_128x128_w4";
            return launch_one<128, 128, 2, 2, true, 4>(a, none, stream);
        case 4:
            tiles(256, 128);
            *name = "gemm_fused_256x128_w8";
            return launch_one<256, 128, 4, 2, true, 5>(a, none, stream);
        case 5:
            tiles(256, 128);
            *name = "gemm_fused_256x128_w8_allcopy";
            return launch_one<256, 128, 4, 2, true, 5, true>(a, none, stream);
        default:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w8";
            return launch_one<256, 256, 2, 4, true, 4>(a, none, stream);
    }
}

hipError_t launch_gemm_splitk(const GemmArgs& a0, const ShrinkArgs& sa, int variant, hipStream_t stream,
                              const char** name)
{
    GemmArgs a = a0;
    auto tiles = [&](int BM, int BN) {
        a.tiles_m = (a.m_end - a.m_begin + BM - 1) / BM;
        a.tiles_n = 0;
        for (int k = 0; k < a.g.n; ++k) {
            a.g.s[k].tile0 = a.tiles_n;
            a.tiles_n += (a.g.s[k].N + BN - 1) / BN;
        }
    };
    switch (variant) {
        case 1:
            tiles(256, 128);
            *name = "gemm_splitk_shrink_256x128_w4";
            return launch_one<256, 128, 2, 2, false, 5>(a, sa, stream);
        case 2:
            tiles(256, 64);
            *name = "gemm_splitk_shrink_256x64_w4";
            return launch_one<256, 64, 4, 1, false, 5>(a, sa, stream);
        case 3:
            tiles(128, 128);
            *name = "gemm_splitk_shrink_128x128_w4";
            return launch_one<128, 128, 2, 2, false, 5>(a, sa, stream);
        case 4:
            tiles(128, 128);
            *name = "gemm_splitk_shrink_128x128_w4_s8";
            return launch_one<128, 128, 2, 2, false, 8>(a, sa, stream);
        default:
            tiles(256, 128);
            *name = "gemm_splitk_shrink_256x128_w8";
            return launch_one<256, 128, 4, 2, false, 5>(a, sa, stream);
    }
}

}  // namespace lora
