// Base projection x W^T on the bf16 matrix cores with the LoRA expand folded into the epilogue
// (paper Sec. 2.2: the adapter's activations are added to the backbone layer's output; Sec. 1: the
// backbone is shared, adapters stay unmerged).
//
// Rows of the GEMM are grouped positions m (token perm[m]); x rows are gathered through perm when the
// tile is staged and output rows are scattered back through it, so `out` is in token order.
//
// Tiling: BM x BN output tile per workgroup, K walked in 64-wide LDS tiles, double buffered; the next
// tile is fetched into registers while the current one feeds the MFMAs.  LDS rows are 128 bytes
// (8 chunks of 16 bytes); chunk c of row rr is stored at position c ^ (rr & 7), which makes both the
// 16-byte row-major writes and the MFMA-layout reads (32 rows x one chunk) bank-conflict free.
//
// MFMA 32x32x16 bf16 with W as the first operand and x as the second: the accumulator of a lane then
// holds one grouped row m (its column index) and, per group of four registers, four consecutive
// output columns n, so results leave as 8-byte (bf16) or 16-byte (fp32) stores.
//
// FUSED: K is walked in full; then for every distinct slot among the 32 rows of an accumulator block
// the shrink result v (scaled, rounded to bf16) and that slot's B rows are fed as extra K steps
// straight from global memory in MFMA layout; result is rounded once to bf16.
// SPLITK: blockIdx selects a K range; fp32 partial tiles are written for the reduce + expand kernel.
#include "lora_internal.hpp"

namespace lora {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int BM, int BN, int WGM, int WGN, bool FUSED>
__global__ __launch_bounds__(WGM * WGN * kWave) void gemm_kernel(GemmArgs a)
{
    constexpr int NT = WGM * WGN * kWave;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wave tile
    constexpr int MB = WTM / 32, NB = WTN / 32;     // 32x32 accumulator blocks per wave
    constexpr int XCH = BM * 8 / NT, WCH = BN * 8 / NT;  // 16-byte chunks per thread per tile
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads");
    static_assert(NT % 8 == 0, "threads");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* sX = smem;                       // [2][BM*64]
    uint16_t* sW = smem + 2 * BM * kBK;        // [2][BN*64]

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

    // global source rows for the staging loads (clamped: rows past T or N are computed, never stored)
    const int ld_chunk = tid & 7, ld_row = tid >> 3;
    const uint16_t* xsrc[XCH];
    const uint16_t* wsrc[WCH];
#pragma unroll
    for (int q = 0; q < XCH; ++q) {
        int m = m0 + ld_row + q * (NT / 8);
        if (m > T - 1) m = T - 1;
        xsrc[q] = a.x + (size_t)a.dv.perm[m] * K + ld_chunk * 8;
    }
#pragma unroll
    for (int q = 0; q < WCH; ++q) {
        int n = n0 + ld_row + q * (NT / 8);
        if (n > N - 1) n = N - 1;
        wsrc[q] = a.W + (size_t)n * K + ld_chunk * 8;
    }

    f32x16 acc[NB][MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

    u32x4 xr[XCH], wr[WCH];
    auto fetch = [&](int kt) {
        const int k0 = kt * kBK;
#pragma unroll
        for (int q = 0; q < XCH; ++q) xr[q] = *reinterpret_cast<const u32x4*>(xsrc[q] + k0);
#pragma unroll
        for (int q = 0; q < WCH; ++q) wr[q] = *reinterpret_cast<const u32x4*>(wsrc[q] + k0);
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int q = 0; q < XCH; ++q) {
            const int rr = ld_row + q * (NT / 8);
            *reinterpret_cast<u32x4*>(sX + buf * BM * kBK + (rr * 8 + (ld_chunk ^ (rr & 7))) * 8) = xr[q];
        }
#pragma unroll
        for (int q = 0; q < WCH; ++q) {
            const int rr = ld_row + q * (NT / 8);
            *reinterpret_cast<u32x4*>(sW + buf * BN * kBK + (rr * 8 + (ld_chunk ^ (rr & 7))) * 8) = wr[q];
        }
    };

    if (kt_begin < kt_end) {
        fetch(kt_begin);
        stage(0);
    }
    __syncthreads();

    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const int buf = (kt - kt_begin) & 1;
        if (kt + 1 < kt_end) fetch(kt + 1);
        const uint16_t* bx = sX + buf * BM * kBK;
        const uint16_t* bw = sW + buf * BN * kBK;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int c = kk * 2 + h;
            bf16x8 wf[NB], xf[MB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int rr = wn * WTN + nb * 32 + i;
                wf[nb] = as_bf16x8(*reinterpret_cast<const u32x4*>(bw + (rr * 8 + (c ^ (rr & 7))) * 8));
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int rr = wm * WTM + mb * 32 + i;
                xf[mb] = as_bf16x8(*reinterpret_cast<const u32x4*>(bx + (rr * 8 + (c ^ (rr & 7))) * 8));
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], xf[mb], acc[nb][mb], 0, 0, 0);
        }
        if (kt + 1 < kt_end) stage(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue ----------------
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m0 + wm * WTM + mb * 32 + i;      // grouped row of this lane
        const bool m_ok = m < T;

        if (FUSED) {
            const int my_slot = m_ok ? a.dv.row_slot[m] : -1;
            unsigned long long todo = __ballot(my_slot >= 0);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const int s = __shfl(my_slot, leader, kWave);
                const unsigned long long peers = __ballot(my_slot == s);
                todo &= ~peers;
                const int r = a.dv.slot_rank[s];
                if (r <= 0) continue;
                const float sc = a.dv.slot_scale[s];
                const uint16_t* Bs = a.dv.slots + (size_t)s * a.dv.slot_stride + a.b_off;
                const bool mine = (my_slot == s);
                for (int kq = 0; kq < r; kq += 16) {
                    const int k = kq + h * 8;
                    const bool k_ok = k < r;
                    // second operand: scaled shrink output of this lane's row, rounded to bf16
                    bf16x8 vf;
                    {
                        f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
                        if (mine && k_ok) {
                            for (int c = 0; c < a.n_kc; ++c) {
                                const float* vp = a.vpart + ((size_t)c * T + m) * a.dv.max_rank + k;
                                lo += *reinterpret_cast<const f32x4*>(vp);
                                hi += *reinterpret_cast<const f32x4*>(vp + 4);
                            }
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            vf[e] = (__bf16)(lo[e] * sc);
                            vf[4 + e] = (__bf16)(hi[e] * sc);
                        }
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int n = n0 + wn * WTN + nb * 32 + i;
                        u32x4 bv = {0u, 0u, 0u, 0u};
                        if (k_ok && n < N) bv = *reinterpret_cast<const u32x4*>(Bs + (size_t)n * r + k);
                        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(bv), vf, acc[nb][mb], 0, 0, 0);
                    }
                }
            }
        }

        if (m_ok) {
            if (FUSED) {
                uint16_t* orow = a.out + (size_t)a.dv.perm[m] * N;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = n0 + wn * WTN + nb * 32 + g * 8 + h * 4;
                        if (n < N) {
                            bf16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[nb][mb][g * 4 + e];
                            *reinterpret_cast<u32x2*>(orow + n) = __builtin_bit_cast(u32x2, o);
                        }
                    }
            } else {
                float* prow = a.part + ((size_t)split * a.Mpad + m) * N;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = n0 + wn * WTN + nb * 32 + g * 8 + h * 4;
                        if (n < N) {
                            f32x4 o = {acc[nb][mb][g * 4 + 0], acc[nb][mb][g * 4 + 1], acc[nb][mb][g * 4 + 2],
                                       acc[nb][mb][g * 4 + 3]};
                            *reinterpret_cast<f32x4*>(prow + n) = o;
                        }
                    }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, bool FUSED>
hipError_t launch_one(const GemmArgs& a, hipStream_t stream)
{
    constexpr int NT = WGM * WGN * kWave;
    constexpr size_t lds = (size_t)2 * (BM + BN) * kBK * sizeof(uint16_t);
    auto kfn = gemm_kernel<BM, BN, WGM, WGN, FUSED>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = a.tiles_m * a.tiles_n * (FUSED ? 1 : a.split_k);
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_fused(const GemmArgs& a0, hipStream_t stream, const char** name)
{
    GemmArgs a = a0;
    constexpr int BM = 256, BN = 256;
    a.tiles_m = (a.dv.T + BM - 1) / BM;
    a.tiles_n = (a.N + BN - 1) / BN;
    *name = "gemm_fused_256x256";
    return launch_one<BM, BN, 2, 4, true>(a, stream);
}

hipError_t launch_gemm_splitk(const GemmArgs& a0, hipStream_t stream, const char** name)
{
    GemmArgs a = a0;
    constexpr int BM = 256, BN = 128;
    a.tiles_m = (a.dv.T + BM - 1) / BM;
    a.tiles_n = (a.N + BN - 1) / BN;
    *name = "gemm_splitk_256x128";
    return launch_one<BM, BN, 4, 2, false>(a, stream);
}

}  // namespace lora
