// Base projection x W^T for small batches (decode), where the weight stream from HBM and the re-read of x
// from L2 bound the kernel (paper Sec. 2.2: the adapter's activations are added to the backbone layer's
// output; Sec. 5.1.2: backbone latency grows linearly with the batch).
//
// Same tiling idea as the 32-wide-K kernel - BM x BN tile per workgroup, tiles copied global -> LDS with
// global_load_lds, MFMA 32x32x16 with W as first operand - but K is walked in 64-wide tiles, so that every
// row segment a copy instruction fetches is one whole 128-byte cache line (eight lanes per line, eight rows
// per instruction).  Measured on a stream of W tiles from HBM mixed with x tiles from L2, whole-line
// segments move 25 - 30 % more bytes per second through a CU's vector cache than 64-byte half lines: with
// half lines every line is requested twice.
//
// LDS rows are 128 bytes; chunk c (16 bytes) of row r sits at position c ^ ((r >> 1) & 7).  The copy engine
// places lane l at byte 16 l of the instruction's 1 KB, so the swizzle is applied on the global side (lane l
// fetches the chunk that belongs at its position; the eight lanes of a row still cover its whole line).  The
// LDS serves a 128-bit read 16 lanes per cycle, the 16 lanes being those of a 32-lane half whose lane-index
// bits 2, 3, 4 have equal parity; among them rows of equal parity differ in (r >> 1) & 7, so the MFMA-layout
// reads (32 rows x one chunk) are bank-conflict free.
//
// Ring of NS stages, one barrier per tile: at the top of iteration j every wave waits for its own copies of
// tile j (younger ones stay in flight), meets the others, refills the stage tile j - 1 has just left with tile
// j + NS - 1, then multiplies tile j.  NS - 1 tiles are in flight behind the one being multiplied.
#include "gemm_epilogue.hpp"

namespace lora {
namespace {

constexpr int kTK64 = 64;    // K extent of one LDS tile (bf16 elements): 128-byte rows
constexpr int kRowB = 128;

__device__ inline void copy16_to_lds(const void* gptr, uint32_t lds_addr)
{
    // issued from inline assembly: the only ordering against later LDS reads is the explicit vmcnt wait +
    // barrier of the main loop
    // m0 carries the LDS address.  It cannot be named as a clobber (a reserved register: the compiler rejects
    // it) and needs none: the compiler keeps no value in m0 between statements, it writes m0 itself directly in
    // front of each instruction of its own that reads it.  Putting the old value back after the copy was tried
    // and stalls every copy (the write to m0 waits until the copy instruction has read it): + 0.2 us per K tile.
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}

// One dword per lane, global -> LDS (lane l lands at lds_addr + 4 l), coherent at device scope: the poll of a
// counter that other workgroups of the launch advance.
__device__ inline void poll4_to_lds(const void* gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off sc1" ::"v"(gptr), "s"(lds_addr) : "memory");
}

template <int N>
__device__ inline void wait_copies_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// GLU (fused path only): the launch serves two projections of the same tokens, gate = slice 0 and up = slice 1, and
// stores silu(gate) * up.  A workgroup then owns BN / 2 output columns; the W part of a stage alternates between
// the two matrices in blocks of 32 rows (block 2 j: rows of gate, block 2 j + 1: the same rows of up), so that a
// wave holds both factors of every output element it owns in the same lane.
template <int BM, int BN, int WGM, int WGN, bool FUSED, int NS, bool GLU = false>
__global__ __launch_bounds__(WGM* WGN* kWave) void gemm_rows128_kernel(GemmArgs a, ShrinkArgs sa)
{
    static_assert(!GLU || FUSED, "the product is formed in the fused epilogue");
    constexpr int NWV = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;           // wave tile
    constexpr int MB = WTM / 32, NB = WTN / 32;             // 32x32 accumulator blocks per wave
    constexpr int STAGE_B = (BM + BN) * kRowB;              // bytes per stage
    constexpr int XQ = BM / 8 / NWV, WQ = BN / 8 / NWV;     // copy instructions (8 rows) per wave and tile
    constexpr int QPT = XQ + WQ;
    static_assert(BM % (8 * NWV) == 0 && BN % (8 * NWV) == 0, "tile/waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    static_assert(NS >= 2 && NS <= 5 && (NS - 1) * QPT <= 63, "stages / vmcnt range");
    static_assert(NS * STAGE_B <= 160 * 1024, "LDS");

    __shared__ __attribute__((aligned(1024))) uint8_t ring[NS * STAGE_B];
    // fused path, shrink inside the launch: the shrink workgroups' counter as polled during the main loop and the
    // verdict for the whole workgroup
    __shared__ uint32_t s_poll[kWave];
    __shared__ uint32_t s_early;
    // split path: the workgroups past the tile grid only do shrink items
    const int extra = (int)gridDim.x - a.main_grid;          // shrink-only workgroups of this launch
    if (!FUSED && sa.on && (int)blockIdx.x >= a.main_grid) {
        const int idx = (int)blockIdx.x - a.main_grid;
        float* sRed = reinterpret_cast<float*>(ring);
        const ShrinkPrefetch pa = shrink_prefetch(sa, idx);
        shrink_block_items<NWV>(sa, idx, extra, extra * a.shrink_q, sRed, pa);
        const int rest = extra * a.shrink_q + (int)blockIdx.x;
        if (rest < pa.n_items) {                              // uniform over the workgroup
            const ShrinkPrefetch pb = shrink_prefetch(sa, rest);
            shrink_block_items<NWV>(sa, rest, gridDim.x, pb.n_items, sRed, pb);
        }
        return;
    }
    // fused path: the workgroups at the front of the grid do the launch's shrink items and report
    const int front = FUSED ? a.shrink_front : 0;
    if (FUSED && front > 0 && (int)blockIdx.x < front) {
        float* sRed = reinterpret_cast<float*>(ring);
        const ShrinkPrefetch pa = shrink_prefetch(sa, blockIdx.x);
        shrink_block_items<NWV>(sa, blockIdx.x, front, pa.n_items, sRed, pa);
        // Every wave orders its stores at workgroup scope and meets the others; one thread then issues the single
        // device-scope release (a write-back of this L2's dirty lines: one per workgroup, not one per wave) and
        // reports.  That the other waves' stores are covered by that one release rests on the hardware (one CU,
        // one L2 behind it, stores of a CU reach the L2 in order), not on the language's memory model.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            atomicAdd(a.sync, 1u);
        }
        return;
    }
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)ring;

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave % WGM, wn = wave / WGM;
    const int T = a.m_end, K = a.K;                         // rows past m_end are computed, never stored

    // blockIdx -> (split, tile_m, tile_n): consecutive blockIdx values land on different XCDs, so the K split
    // is the fastest index on the split path (every XCD keeps one x K-range in its L2)
    int split = 0, tile_m, tile_n;
    {
        int b = (int)blockIdx.x - front;
        if (!FUSED) {
            split = b % a.split_k;
            b /= a.split_k;
        }
        tile_m = b % a.tiles_m;
        tile_n = b / a.tiles_m;
    }
    int si = 0;
    if (!GLU)
        for (int k = 1; k < a.g.n; ++k)
            if (tile_n >= a.g.s[k].tile0) si = k;
    const Slice sl = pick_slice(a.g, si);
    const uint16_t* const xg = sl.x;
    const uint16_t* const Wg = sl.W;
    const uint16_t* const Wup = GLU ? a.g.s[1].W : sl.W;
    const int N = sl.N;
    // n0: first column inside the slice (GLU: first output column; the tile is BN / 2 of them wide)
    const int m0 = a.m_begin + tile_m * BM, n0 = (tile_n - sl.tile0) * (GLU ? BN / 2 : BN);

    ShrinkPrefetch spf{};
    const int rest_first = extra * a.shrink_q + (int)blockIdx.x;     // this workgroup's first item after its tile
    if (!FUSED && sa.on) spf = shrink_prefetch(sa, rest_first);

    const int kt_total = K / kTK64;
    int kt_begin = 0, kt_end = kt_total;
    if (!FUSED) {
        kt_begin = (int)((long long)kt_total * split / a.split_k);
        kt_end = (int)((long long)kt_total * (split + 1) / a.split_k);
    }
    const int nk = kt_end - kt_begin;

    // Copy assignment: instruction q of wave w fills stage rows 8 (w XQ + q) .. + 7 of the x part (same for
    // the W part with WQ); lane l owns row l / 8 of those and chunk position l % 8.  Rows past T or N are
    // clamped to the last valid row: they are computed, never stored.
    uint32_t xoff[XQ], woff[WQ];                            // element offsets of this lane's 16 bytes in tile 0
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        const int r = (wave * XQ + q) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int m = m0 + r;
        if (m > T - 1) m = T - 1;
        xoff[q] = (uint32_t)a.dv.perm[m] * (uint32_t)K + (uint32_t)(c * 8 + kt_begin * kTK64);
    }
    bool w_up[WQ];                                           // GLU: this copy instruction's rows come from `up` (uniform over the wave)
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int r = (wave * WQ + q) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int n = GLU ? n0 + (r >> 6) * 32 + (r & 31) : n0 + r;
        if (n > N - 1) n = N - 1;
        woff[q] = (uint32_t)n * (uint32_t)K + (uint32_t)(c * 8 + kt_begin * kTK64);
        w_up[q] = GLU && ((((wave * WQ + q) * 8) >> 5) & 1);
    }
    const uint32_t cp_x = ring_addr + wave * XQ * 1024;
    const uint32_t cp_w = ring_addr + BM * kRowB + wave * WQ * 1024;
    // copy instructions [q_begin, q_end) of tile t of this workgroup's K range; the W rows (from HBM) go first
    auto copy_part = [&](int t, int stage, int q_begin, int q_end) {
        const uint32_t k0 = (uint32_t)t * kTK64, so = (uint32_t)stage * STAGE_B;
#pragma unroll
        for (int q = 0; q < QPT; ++q) {
            if (q < q_begin || q >= q_end) continue;
            if (q < WQ)
                copy16_to_lds((w_up[q] ? Wup : Wg) + (woff[q] + k0), __builtin_amdgcn_readfirstlane(cp_w + so + q * 1024));
            else
                copy16_to_lds(xg + (xoff[q - WQ] + k0), __builtin_amdgcn_readfirstlane(cp_x + so + (q - WQ) * 1024));
        }
    };
    auto copy_tile = [&](int t, int stage) { copy_part(t, stage, 0, QPT); };

    f32x16 acc[MB][NB];
    init_accumulators<MB, NB, FUSED && !GLU>(acc, sl, n0 + wn * WTN);       // GLU: no bias (refused by the host)

    // byte offset of this lane's fragment of K step kk inside a 32-row block: row i, chunk 2 kk + h
    const int sw = (i >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) rd[kk] = i * kRowB + (((2 * kk + h) ^ sw) << 4);
    const int x_base = wm * WTM * kRowB, w_base = (BM + wn * WTN) * kRowB;

    // prologue: tiles 0 .. NS - 2
#pragma unroll
    for (int d = 0; d < NS - 1; ++d)
        if (d < nk) copy_tile(d, d);

    // fused path: the epilogue's per-row data travels while the first tiles do
    constexpr bool PRE = FUSED && MB <= 2 && !GLU;
    TilePrefetch<PRE ? MB : 1> pre;
    if constexpr (PRE) {
        prefetch_rows(pre, a, m0 + wm * WTM);
        if (front == 0) prefetch_v_issue(pre, a, sl, m0 + wm * WTM);      // else: not there yet
    }
    // Shrink inside the launch: the tile workgroups need its results only in the epilogue.  The counter of the
    // shrink workgroups is polled four tiles before the end (a copy into LDS, ordered like the tile copies: it
    // has landed when tile nk - 2 has); two tiles before the end one thread reads the verdict, makes the shrink
    // results visible and publishes it; during the last tile every wave requests its shares of the results.
    // When the poll came too early the wait after the loop takes over.
    bool early = false;
    const bool poll_on = PRE && front > 0 && nk >= 4;
    const uint32_t poll_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)s_poll;
    // Past the wait for the shrink workgroups every tile workgroup takes a ticket; the one with the last ticket
    // sets the two counters back to zero for the next launch (at the end of the kernel: nobody of this launch
    // looks at them any more).  The ticket is requested here and read only then, so that nobody waits for it.
    uint32_t ticket = 0;
    bool have_ticket = false;                                // thread 0 only
    auto passed_the_wait = [&]() {
        ticket = atomicAdd(a.sync + 1, 1u);
        have_ticket = true;
        // what the shrink workgroups wrote is read from here on: drop what this CU and this L2 may hold of it
        // (the acquire side; no wait for older loads is needed, the poll that showed the counter has landed)
        asm volatile("buffer_inv sc1" ::: "memory");
    };

    // Software pipeline.  The fragments of a K step are read one step ahead, also across tiles: the barrier that
    // makes tile j + 1 complete for every wave (and frees the stage of tile j, whose last fragments are in
    // registers by then) sits in front of the MFMAs of tile j's last K step, and the first fragments of tile j + 1
    // are requested right behind it, so that those MFMAs cover the LDS latency.  With the barrier at the top of a
    // tile every wave of the workgroup would wait out that latency at the same time, with no MFMA in flight.
    // Tile j + NS - 1 goes into the stage tile j - 1 has left, its copy instructions spread over the first
    // three K steps of tile j (a wave that is held at a copy instruction by a full memory pipeline cannot issue
    // its MFMAs meanwhile); all of them are out when the wave waits for tile j + 1.
    // own copies of tile t landed (the at most NS - 2 younger tiles stay in flight), then the barrier
    auto wait_for_tile = [&](int t) {
        int young = nk - 1 - t;
        if (young > NS - 2) young = NS - 2;
        if (young >= 3) wait_copies_then_barrier<(NS >= 5 ? 3 : 0) * QPT>();
        else if (young == 2) wait_copies_then_barrier<(NS >= 4 ? 2 : 0) * QPT>();
        else if (young == 1) wait_copies_then_barrier<QPT>();
        else wait_copies_then_barrier<0>();
    };
    // what the fused path does behind the barrier of tile t (see above: poll, verdict, request)
    auto behind_barrier = [&](int t) {
        if constexpr (PRE) {
            if (poll_on) {
                if (t == nk - 4 && wave == 0) poll4_to_lds(a.sync, __builtin_amdgcn_readfirstlane(poll_addr));
                if (t == nk - 2 && threadIdx.x == 0) {
                    const bool done = s_poll[0] >= (uint32_t)a.front_expect;     // landed: older than the copies the wait let pass
                    if (done) passed_the_wait();
                    s_early = done ? 1u : 0u;
                }
                if (t == nk - 1) {
                    early = s_early != 0u;
                    if (early) prefetch_v_issue(pre, a, sl, m0 + wm * WTM);
                }
            }
        }
    };
    bf16x8 Fw[2][NB], Fx[2][MB];
    auto read_step = [&](int f, const uint8_t* st, int kk) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            Fw[f][nb] = as_bf16x8(*reinterpret_cast<const u32x4*>(st + w_base + nb * 32 * kRowB + rd[kk]));
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            Fx[f][mb] = as_bf16x8(*reinterpret_cast<const u32x4*>(st + x_base + mb * 32 * kRowB + rd[kk]));
    };
    if (nk > 0) {
        wait_for_tile(0);
        behind_barrier(0);
        read_step(0, ring, 0);
    }
    int cur = 0, fre = NS - 1;                               // stages of tile j and of tile j - 1
    for (int j = 0; j < nk; ++j) {
        const bool refill = j + NS - 1 < nk;
        const uint8_t* st = ring + cur * STAGE_B;
        const int nxt = (cur + 1 == NS) ? 0 : cur + 1;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) {
                read_step((kk + 1) & 1, st, kk + 1);
                if (refill) copy_part(j + NS - 1, fre, kk * QPT / 3, (kk + 1) * QPT / 3);
            } else if (j + 1 < nk) {
                // this wave's last fragments of tile j are in registers before it lets the others refill the stage
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                wait_for_tile(j + 1);
                behind_barrier(j + 1);
                read_step(0, ring + nxt * STAGE_B, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = mfma32(Fw[kk & 1][nb], Fx[kk & 1][mb], acc[mb][nb]);
        }
        fre = cur;
        cur = nxt;
    }

    // ---------------- epilogue ----------------
    static_assert(!FUSED || NS * STAGE_B >= NWV * epilogue_bytes_per_wave<NB>(), "ring too small for the fused epilogue");
    static_assert(!GLU || NS * STAGE_B >= NWV * glu_epilogue_bytes_per_wave(), "ring too small for the gated epilogue");
    static_assert(FUSED || NS * STAGE_B >= NWV * kRedFloatsPerWave * 4, "ring too small for the reduction");
    if (FUSED) __syncthreads();
    if (FUSED && front > 0 && !early) {                           // uniform over the workgroup
        // The shrink results come from the workgroups at the front of this launch.  They hold the lowest
        // indices, so they were dispatched before this workgroup and never wait for anything: the wait ends.
        // It is bounded all the same; if it expires the call's result is invalid and flagged.
        if (threadIdx.x == 0) {
            int spins = 0;
            while (__hip_atomic_load(a.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)a.front_expect) {
                if (++spins > a.wait_spins) {
                    atomicOr(a.flags, kFlagInternal);
                    break;
                }
                __builtin_amdgcn_s_sleep(32);
            }
            passed_the_wait();
        }
        __syncthreads();
        if constexpr (PRE) prefetch_v_issue(pre, a, sl, m0 + wm * WTM);
    }
    if constexpr (PRE) prefetch_v_finish(pre, a, sl, m0 + wm * WTM);
    if constexpr (GLU)
        finish_tile_glu<MB, NB>(acc, a, sl, a.g.s[1], m0 + wm * WTM, n0 + wn * (WTN / 2), wave, reinterpret_cast<uint16_t*>(ring));
    else if constexpr (PRE)
        finish_tile_prefetched<MB, NB>(acc, a, sl, m0 + wm * WTM, n0 + wn * WTN, wave, reinterpret_cast<uint16_t*>(ring), pre);
    else
        finish_tile<MB, NB, FUSED>(acc, a, sl, m0 + wm * WTM, n0 + wn * WTN, split, wave, reinterpret_cast<uint16_t*>(ring));
    if (!FUSED && sa.on) {
        __syncthreads();
        shrink_block_items<NWV>(sa, rest_first, gridDim.x, spf.n_items, reinterpret_cast<float*>(ring), spf);
    }
    if (FUSED) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy of this wave is still on its way
    if (FUSED && have_ticket && ticket == gridDim.x - (uint32_t)front - 1u) {
        __hip_atomic_store(a.sync, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.sync + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int BM, int BN, int WGM, int WGN, bool FUSED, int NS, bool GLU = false>
hipError_t launch_rows128(GemmArgs a, const ShrinkArgs& sa, hipStream_t stream)
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
    int grid = a.tiles_m * a.tiles_n * (FUSED ? 1 : a.split_k);
    const int extra = FUSED ? 0 : a.main_grid;            // on entry: workgroups that only do shrink items
    a.main_grid = grid;
    grid += extra;
    if (FUSED) grid += a.shrink_front;                    // those come first
    hipLaunchKernelGGL((gemm_rows128_kernel<BM, BN, WGM, WGN, FUSED, NS, GLU>), dim3(grid), dim3(WGM * WGN * kWave), 0,
                       stream, a, sa);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_rows128_fused(const GemmArgs& a, const ShrinkArgs& none, int variant, hipStream_t stream,
                                     const char** name)
{
    // `none`: the shrink work of the launch when a.shrink_front > 0, otherwise unused
    switch (variant) {
        case 1:
            *name = "gemm_fused_128x128x64_w4";
            return launch_rows128<128, 128, 2, 2, true, 4>(a, none, stream);
        case 2:
            *name = "gemm_fused_256x256x64_w8";
            return launch_rows128<256, 256, 2, 4, true, 2>(a, none, stream);
        case 3:
            *name = "gemm_fused_256x192x64_w8";
            return launch_rows128<256, 192, 4, 2, true, 2>(a, none, stream);
        case 4:
            *name = "gemm_fused_256x128x64_w4";
            return launch_rows128<256, 128, 2, 2, true, 3>(a, none, stream);
        case 5:
            *name = "gemm_fused_256x256x64_w4";
            return launch_rows128<256, 256, 2, 2, true, 2>(a, none, stream);
        default:
            *name = "gemm_fused_256x128x64_w8";
            return launch_rows128<256, 128, 4, 2, true, 3>(a, none, stream);
    }
}

hipError_t launch_gemm_rows128_glu(const GemmArgs& a, const ShrinkArgs& none, int variant, hipStream_t stream,
                                   const char** name)
{
    if (variant == 1) {
        *name = "gemm_glu_128x128x64_w4";
        return launch_rows128<128, 128, 2, 2, true, 4, true>(a, none, stream);
    }
    *name = "gemm_glu_256x128x64_w8";
    return launch_rows128<256, 128, 4, 2, true, 3, true>(a, none, stream);
}

hipError_t launch_gemm_rows128_splitk(const GemmArgs& a, const ShrinkArgs& sa, int variant, hipStream_t stream,
                                      const char** name)
{
    switch (variant) {
        case 1:
            *name = "gemm_splitk_shrink_128x128x64_w4";
            return launch_rows128<128, 128, 2, 2, false, 4>(a, sa, stream);
        case 2:
            *name = "gemm_splitk_shrink_256x128x64_w4";
            return launch_rows128<256, 128, 2, 2, false, 3>(a, sa, stream);
        default:
            *name = "gemm_splitk_shrink_256x128x64_w8";
            return launch_rows128<256, 128, 4, 2, false, 3>(a, sa, stream);
    }
}

}  // namespace lora
