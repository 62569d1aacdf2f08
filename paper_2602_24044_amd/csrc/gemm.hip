// Base projection x W^T on the bf16 matrix cores (paper Sec. 2.2: the adapter's activations are added
// to the backbone layer's output; Sec. 1: the backbone is shared, adapters stay unmerged).
//
// Rows of the GEMM are grouped positions m (token perm[m]); x rows are gathered through perm when the
// tile is staged and output rows are scattered back through it, so `out` is in token order.
//
// Tiling: BM x BN output tile per workgroup, K walked in 64-wide tiles through two LDS stages.  Tiles
// are copied global -> LDS directly (global_load_lds, 16 bytes per lane, no staging registers and no
// LDS store instructions): one wave instruction fills 1 KB = 8 LDS rows of 128 bytes.  Chunk c (16
// bytes) of row rr is kept at position c ^ (rr & 7); because the copy engine places lane l at byte
// 16 l of the wave's 1 KB, the swizzle is applied on the global side (lane l fetches the chunk that
// belongs at its position).  The MFMA-layout reads (32 rows x one chunk) are then bank-conflict free.
// The copy of tile j + 2 is issued as soon as every wave has finished reading tile j and is in
// flight during the whole of tile j + 1 (see the main loop for the schedule).
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
#include "device_common.hpp"

#include <type_traits>
#include <utility>

namespace lora {
namespace {

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

template <int BM, int BN, int WGM, int WGN, bool FUSED, int D>
__global__ __launch_bounds__(WGM * WGN * kWave) void gemm_kernel(GemmArgs a, ShrinkArgs sa)
{
    constexpr int NT = WGM * WGN * kWave;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wave tile
    constexpr int MB = WTM / 32, NB = WTN / 32;     // 32x32 accumulator blocks per wave
    constexpr int XCH = BM * 8 / NT, WCH = BN * 8 / NT;  // 16-byte chunks per thread per tile
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads");

    // one static array per stage and operand: distinct objects let the compiler keep copies into one
    // stage in flight while the other stage is being read
    __shared__ __attribute__((aligned(1024))) uint16_t sX0[BM * kBK];
    __shared__ __attribute__((aligned(1024))) uint16_t sX1[BM * kBK];
    __shared__ __attribute__((aligned(1024))) uint16_t sW0[BN * kBK];
    __shared__ __attribute__((aligned(1024))) uint16_t sW1[BN * kBK];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave % WGM, wn = wave / WGM;
    const int T = a.dv.T, N = a.N, K = a.K;

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
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int kt_total = K / kBK;
    int kt_begin = 0, kt_end = kt_total;
    if (!FUSED) {
        kt_begin = (int)((long long)kt_total * split / a.split_k);
        kt_end = (int)((long long)kt_total * (split + 1) / a.split_k);
    }
    const int nk = kt_end - kt_begin;

    // Copy assignment: wave instruction q of wave w fills LDS rows 8 (w XQ + q) .. + 7 of the X tile
    // (same for W with WQ); lane l owns row l / 8 of those and chunk position l % 8.  Rows past T or N are
    // clamped to the last valid row: they are computed, never stored.
    constexpr int NWV = NT / kWave;
    constexpr int XQ = BM / 8 / NWV, WQ = BN / 8 / NWV;     // wave instructions per stage
    static_assert(BM % (8 * NWV) == 0 && BN % (8 * NWV) == 0, "tile/waves");
    const int cp_row = lane >> 3;
    const int cp_chunk = (lane & 7) ^ cp_row;               // (row & 7) == cp_row: row blocks start at multiples of 8
    uint32_t xoff[XQ], woff[WQ];                            // element offsets of this lane's 16 bytes at k = 0
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
        int m = m0 + (wave * XQ + q) * 8 + cp_row;
        if (m > T - 1) m = T - 1;
        xoff[q] = (uint32_t)a.dv.perm[m] * (uint32_t)K + (uint32_t)(cp_chunk * 8 + kt_begin * kBK);
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        int n = n0 + (wave * WQ + q) * 8 + cp_row;
        if (n > N - 1) n = N - 1;
        woff[q] = (uint32_t)n * (uint32_t)K + (uint32_t)(cp_chunk * 8 + kt_begin * kBK);
    }

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    // ---- software-pipelined main loop ----
    // State at the top of iteration j: tile j is complete in stage j & 1, the fragments of its first K
    // step are in F[0], and the copy of tile j + 1 into the other stage is in flight.  Each K step issues
    // the LDS reads of the following step before its own MFMAs.  The single barrier of the iteration
    // sits between K step 2 and 3: every wave has then read all of tile j (its last fragments are in
    // registers) and its own share of tile j + 1 has landed, so after the barrier tile j + 1 is complete
    // for everyone and stage j & 1 is free: the copy of tile j + 2 starts there, the first fragments of
    // tile j + 1 are read, and the MFMAs of step 3 cover the barrier skew and the LDS latency.
    bf16x8 Fw[2][NB], Fx[2][MB];
    auto copy_tile = [&](auto st_c, int j) {
        constexpr int ST = decltype(st_c)::value;
        uint16_t* dx = ST ? sX1 : sX0;
        uint16_t* dw = ST ? sW1 : sW0;
        const uint32_t k0 = (uint32_t)j * kBK;
#pragma unroll
        for (int q = 0; q < XQ; ++q)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(a.x + (xoff[q] + k0)),
                (__attribute__((address_space(3))) void*)(dx + (wave * XQ + q) * 512), 16, 0, 0);
#pragma unroll
        for (int q = 0; q < WQ; ++q)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(a.W + (woff[q] + k0)),
                (__attribute__((address_space(3))) void*)(dw + (wave * WQ + q) * 512), 16, 0, 0);
    };
    auto read_frags = [&](auto f_c, auto st_c, int kk) {
        constexpr int Fi = decltype(f_c)::value;
        constexpr int ST = decltype(st_c)::value;
        const uint16_t* bx = ST ? sX1 : sX0;
        const uint16_t* bw = ST ? sW1 : sW0;
        const int c = kk * 2 + h;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int rr = wn * WTN + nb * 32 + i;
            Fw[Fi][nb] = as_bf16x8(*reinterpret_cast<const u32x4*>(bw + (rr * 8 + (c ^ (rr & 7))) * 8));
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int rr = wm * WTM + mb * 32 + i;
            Fx[Fi][mb] = as_bf16x8(*reinterpret_cast<const u32x4*>(bx + (rr * 8 + (c ^ (rr & 7))) * 8));
        }
    };
    auto mma = [&](auto f_c) {
        constexpr int Fi = decltype(f_c)::value;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = mfma32(Fw[Fi][nb], Fx[Fi][mb], acc[mb][nb]);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    auto iteration = [&](auto par_c, int j) {
        constexpr int PAR = decltype(par_c)::value;
        using Cur = std::integral_constant<int, PAR>;
        using Oth = std::integral_constant<int, PAR ^ 1>;
        read_frags(I1{}, Cur{}, 1);
        mma(I0{});
        read_frags(I0{}, Cur{}, 2);
        mma(I1{});
        read_frags(I1{}, Cur{}, 3);
        mma(I0{});
        __syncthreads();
        if (j + 2 < nk) copy_tile(Cur{}, j + 2);
        if (j + 1 < nk) read_frags(I0{}, Oth{}, 0);
        mma(I1{});
    };

    if (nk > 0) {
        copy_tile(I0{}, 0);
        __syncthreads();
        if (nk > 1) copy_tile(I1{}, 1);
        read_frags(I0{}, I0{}, 0);
    }
    for (int j = 0; j < nk; j += 2) {
        iteration(I0{}, j);
        if (j + 1 < nk) iteration(I1{}, j + 1);
    }

    // ---------------- epilogue ----------------
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m0 + wm * WTM + mb * 32 + i;      // grouped row of this lane
        const bool m_ok = m < T;
        const int n_first = n0 + wn * WTN;

        if (FUSED) {
            const int my_slot = m_ok ? a.dv.row_slot[m] : -1;
            const int my_rank = m_ok ? a.dv.row_rank[m] : 0;
            const float my_scale = m_ok ? a.dv.row_scale[m] : 0.f;
            VFromGlobal vs{a.vpart, a.n_kc, T, a.dv.max_rank, m};
            expand_window<NB>(acc[mb], my_slot, my_rank, my_scale, n_first, N, a.dv, a.b_off, vs);
        }

        if (m_ok) {
            if (FUSED) {
                uint16_t* orow = a.out + (size_t)a.dv.perm[m] * N;
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
                const int nblk = (N + 31) / 32;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int bn = (n_first + nb * 32) / 32;
                    if (bn < nblk) {
                        float* blk = a.part + (((size_t)split * (a.Mpad / 32) + (size_t)(m / 32)) * nblk + bn) * 1024;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            f32x4 o = {acc[mb][nb][g * 4 + 0], acc[mb][nb][g * 4 + 1], acc[mb][nb][g * 4 + 2],
                                       acc[mb][nb][g * 4 + 3]};
                            *reinterpret_cast<f32x4*>(blk + g * 256 + i * 8 + h * 4) = o;
                        }
                    }
                }
            }
        }
    }

    // split path: this workgroup's share of the shrink work items of the same projection
    if (!FUSED) {
        __shared__ __attribute__((aligned(16))) float sRed[(FUSED ? 1 : NT / kWave) * kRedFloatsPerWave];
        if (sa.vpart != nullptr) shrink_block_items<NT / kWave>(sa, blockIdx.x, gridDim.x, sRed);
    }
}

template <int BM, int BN, int WGM, int WGN, bool FUSED, int D>
hipError_t launch_one(const GemmArgs& a, const ShrinkArgs& sa, hipStream_t stream)
{
    constexpr int NT = WGM * WGN * kWave;
    auto kfn = gemm_kernel<BM, BN, WGM, WGN, FUSED, D>;
    const int grid = a.tiles_m * a.tiles_n * (FUSED ? 1 : a.split_k);
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), 0, stream, a, sa);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_fused(const GemmArgs& a0, int variant, hipStream_t stream, const char** name)
{
    GemmArgs a = a0;
    ShrinkArgs none{};
    auto tiles = [&](int BM, int BN) {
        a.tiles_m = (a.dv.T + BM - 1) / BM;
        a.tiles_n = (a.N + BN - 1) / BN;
    };
    switch (variant) {
        case 1:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w4";
            return launch_one<256, 256, 2, 2, true, 1>(a, none, stream);
        case 2:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w4_d2";
            return launch_one<256, 256, 2, 2, true, 2>(a, none, stream);
        case 3:
            tiles(128, 128);
            *name = "gemm_fused_128x128_w4_d3";
            return launch_one<128, 128, 2, 2, true, 3>(a, none, stream);
        default:
            tiles(256, 256);
            *name = "gemm_fused_256x256_w8";
            return launch_one<256, 256, 2, 4, true, 1>(a, none, stream);
    }
}

hipError_t launch_gemm_splitk(const GemmArgs& a0, const ShrinkArgs& sa, int variant, hipStream_t stream,
                              const char** name)
{
    GemmArgs a = a0;
    auto tiles = [&](int BM, int BN) {
        a.tiles_m = (a.dv.T + BM - 1) / BM;
        a.tiles_n = (a.N + BN - 1) / BN;
    };
    switch (variant) {
        case 1:
            tiles(256, 128);
            *name = "gemm_splitk_shrink_256x128_w4";
            return launch_one<256, 128, 2, 2, false, 2>(a, sa, stream);
        case 2:
            tiles(256, 64);
            *name = "gemm_splitk_shrink_256x64_w4";
            return launch_one<256, 64, 4, 1, false, 2>(a, sa, stream);
        case 3:
            tiles(128, 128);
            *name = "gemm_splitk_shrink_128x128_w4";
            return launch_one<128, 128, 2, 2, false, 2>(a, sa, stream);
        default:
            tiles(256, 128);
            *name = "gemm_splitk_shrink_256x128_w8";
            return launch_one<256, 128, 4, 2, false, 3>(a, sa, stream);
    }
}

}  // namespace lora
