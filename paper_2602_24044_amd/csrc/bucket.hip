// Token -> adapter segment map (integer only) and the small slot-metadata kernels.
//
// A serving step batches requests of different adapters together (paper Sec. 2.2) and mixes
// prefill chunks with one-token decode requests (Sec. 2.1).  The map groups the tokens of a step
// by the slot their adapter occupies so that each adapter's A and B are streamed once per step.
// SORTED: stable counting sort of token indices by slot; RUNS: token order kept, runs of equal
// slot.  One 1024-thread workgroup: LDS histogram, LDS prefix scan, wavefront ballots for the
// stable rank of a token among equal keys.  RUNS above 4096 tokens: one workgroup per 1024 tokens, two launches.
#include "lora_internal.hpp"

namespace lora {
namespace {

constexpr int kBT = 1024;
constexpr int kNW = kBT / kWave;
constexpr int kMaxKeys = kMaxSlots + 1;

__device__ inline int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive prefix of one int per thread over the workgroup; *total = sum over all threads.
__device__ inline int block_excl_scan(int v, int* s_wave, int* total)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    const int inc = wave_incl_scan(v, lane);
    if (lane == kWave - 1) s_wave[w] = inc;
    __syncthreads();
    if (w == 0) {
        int t = lane < kNW ? s_wave[lane] : 0;
        int ti = wave_incl_scan(t, lane);
        if (lane < kNW) s_wave[lane] = ti - t;
        if (lane == kNW - 1) s_wave[kNW] = ti;
    }
    __syncthreads();
    const int res = s_wave[w] + inc - v;
    *total = s_wave[kNW];
    __syncthreads();
    return res;
}

// Run-length encoding of row_slot[0..T); with align > 0 a run also ends at every multiple of align.  m_start /
// m_slot (may be NULL): copies of the outputs in LDS for the next phase of the same workgroup.
__device__ void rle(const int32_t* row_slot, int T, int align, int32_t* out_start, int32_t* out_slot,
                    int32_t* out_n, int* s_wave, int* m_start, int* m_slot)
{
    int running = 0;
    for (int c = 0; c < T; c += kBT) {
        const int m = c + (int)threadIdx.x;
        int head = 0, s = 0;
        if (m < T) {
            s = row_slot[m];
            head = (m == 0) || (align > 0 && (m % align) == 0) || (row_slot[m - 1] != s);
        }
        int total;
        const int ex = block_excl_scan(head, s_wave, &total);
        if (head) {
            out_start[running + ex] = m;
            out_slot[running + ex] = s;
            if (m_start) {
                m_start[running + ex] = m;
                m_slot[running + ex] = s;
            }
        }
        running += total;
    }
    if (threadIdx.x == 0) {
        out_start[running] = T;
        if (m_start) m_start[running] = T;
        *out_n = running;
    }
}

// Steps of up to kFastT tokens keep every intermediate array in LDS (keys in registers, grouped slots, the
// piece list, the slot tables): the kernel is a chain of dependent phases, and a phase that reads back from
// global memory what the previous one wrote pays a memory round trip each time.
constexpr int kFastT = 4096;
constexpr int kFastPieces = kFastT + kFastT / kPieceRows + 2;

__global__ __launch_bounds__(kBT) void bucket_kernel(BucketArgs a)
{
    __shared__ int s_run[kMaxKeys];      // histogram, then running output offset per key
    __shared__ int s_wave[kNW + 1];
    __shared__ int s_row[kFastT];        // fast path: row_slot
    __shared__ int s_pstart[kFastPieces + 1];
    __shared__ int s_pslot[kFastPieces];
    __shared__ int s_rank[kMaxKeys];     // fast path: slot tables
    __shared__ int s_loc[kMaxKeys];
    __shared__ float s_scale[kMaxKeys];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int T = a.T;
    const int nkeys = a.n_slots + 1;     // key = slot + 1, key 0 = backbone only
    const bool sorted = (a.mode == 0);
    const bool fast = T <= kFastT;
    constexpr int kFastChunks = kFastT / kBT;

    for (int k = tid; k < nkeys; k += kBT) s_run[k] = 0;
    if (fast) {
        for (int k = tid; k < a.n_slots; k += kBT) {
            s_rank[k] = a.slot_rank[k];
            s_loc[k] = a.slot_loc[k];
            s_scale[k] = a.slot_scale[k];
        }
    }
    __syncthreads();

    // keys, histogram, residency check
    bool bad = false;
    int keyreg[kFastChunks];
#pragma unroll
    for (int c = 0; c < kFastChunks; ++c) keyreg[c] = 0;
    auto key_of = [&](int t) {
        const int id = a.ids[t];
        int key = 0;
        if (id >= 0) {
            int s = -1;
            if (id < a.n_ids) s = a.id2slot[id];
            if (s >= 0 && s < a.n_slots) key = s + 1; else bad = true;
        }
        return key;
    };
    if (fast) {
#pragma unroll
        for (int c = 0; c < kFastChunks; ++c) {
            const int t = c * kBT + tid;
            if (t < T) {
                const int key = key_of(t);
                keyreg[c] = key;
                if (sorted) {
                    atomicAdd(&s_run[key], 1);
                } else {
                    a.perm[t] = t;
                    a.row_slot[t] = key - 1;
                    s_row[t] = key - 1;
                }
            }
        }
    } else {
        for (int t = tid; t < T; t += kBT) {
            const int key = key_of(t);
            if (sorted) {
                a.tok_key[t] = key;
                atomicAdd(&s_run[key], 1);
            } else {
                a.perm[t] = t;
                a.row_slot[t] = key - 1;
            }
        }
    }
    if (bad) atomicOr(a.flags, 1u);
    __syncthreads();

    if (sorted) {
        // exclusive scan of the histogram: s_run[key] becomes the first grouped position of key
        int carry = 0;
        for (int k0 = 0; k0 < nkeys; k0 += kBT) {
            const int k = k0 + tid;
            const int c = (k < nkeys) ? s_run[k] : 0;
            int total;
            const int ex = block_excl_scan(c, s_wave, &total);
            if (k < nkeys) s_run[k] = carry + ex;
            carry += total;
        }
        __syncthreads();

        // stable scatter: tokens are taken 1024 at a time in index order, wave after wave
        const int nbits = 32 - __clz(a.n_slots);
        int chunk = 0;
        for (int c = 0; c < T; c += kBT, ++chunk) {
            const int t = c + tid;
            const bool valid = t < T;
            int key = 0;
            if (fast) {
#pragma unroll
                for (int q = 0; q < kFastChunks; ++q)
                    if (q == chunk) key = keyreg[q];
            } else if (valid) {
                key = a.tok_key[t];
            }
            unsigned long long peers = __ballot(valid);
            for (int b = 0; b < nbits; ++b) {
                const bool bit = (key >> b) & 1;
                const unsigned long long mb = __ballot(valid && bit);
                peers &= bit ? mb : ~mb;
            }
            const int rank = __popcll(peers & ((1ull << lane) - 1ull));
            const int cw = __popcll(peers);
            const int rem = T - c;
            const int nw = rem >= kBT ? kNW : (rem + kWave - 1) / kWave;
            for (int w = 0; w < nw; ++w) {
                if (wave == w && valid) {
                    const int pos = s_run[key] + rank;
                    a.perm[pos] = t;
                    a.row_slot[pos] = key - 1;
                    if (fast) s_row[pos] = key - 1;
                }
                __builtin_amdgcn_wave_barrier();
                if (wave == w && valid && rank == cw - 1) s_run[key] += cw;
                __syncthreads();
            }
        }
    }
    __syncthreads();

    // per-row adapter metadata, so that the projection kernels never chase slot -> rank / scale
    const int32_t* rs = fast ? s_row : a.row_slot;
    for (int m = tid; m < T; m += kBT) {
        const int s = rs[m];
        if (fast) {
            a.row_rank[m] = s >= 0 ? s_rank[s] : 0;
            a.row_loc[m] = s >= 0 ? s_loc[s] : -1;
            a.row_scale[m] = s >= 0 ? s_scale[s] : 0.f;
        } else {
            a.row_rank[m] = s >= 0 ? a.slot_rank[s] : 0;
            a.row_loc[m] = s >= 0 ? a.slot_loc[s] : -1;
            a.row_scale[m] = s >= 0 ? a.slot_scale[s] : 0.f;
        }
    }

    rle(rs, T, 0, a.seg_start, a.seg_slot, a.n_seg, s_wave, nullptr, nullptr);
    rle(rs, T, kPieceRows, a.piece_start, a.piece_slot, a.n_pieces, s_wave, fast ? s_pstart : nullptr,
        fast ? s_pslot : nullptr);
    __syncthreads();

    // one 16-byte record per piece for the shrink work loop
    const int n_pieces = *a.n_pieces;
    for (int p = tid; p < n_pieces; p += kBT) {
        int begin, end, s, r, loc;
        if (fast) {
            begin = s_pstart[p];
            end = s_pstart[p + 1];
            s = s_pslot[p];
            r = s >= 0 ? s_rank[s] : 0;
            loc = s >= 0 ? s_loc[s] : -1;
        } else {
            begin = a.piece_start[p];
            end = a.piece_start[p + 1];
            s = a.piece_slot[p];
            r = s >= 0 ? a.slot_rank[s] : 0;
            loc = s >= 0 ? a.slot_loc[s] : -1;
        }
        int4 rec;
        rec.x = begin;
        rec.y = end - begin;
        rec.z = loc;
        rec.w = r;
        reinterpret_cast<int4*>(a.piece_info)[p] = rec;
    }
}

// RUNS mode above kFastT tokens (a prefill batch).  The order is the token order, so everything but the numbering of
// the segments and pieces depends on a token and its predecessor only: one workgroup per kBT tokens, in two
// launches.  The first writes the per-row tables and counts the heads of segments and pieces in its chunk
// (a.tok_key[2 c], [2 c + 1]: the array is unused in this mode); the second numbers them from the counts of the
// chunks in front.  A piece ends at every multiple of kPieceRows, which every chunk boundary is, so no piece
// spans two chunks.
__device__ inline int runs_key(const BucketArgs& a, int t, bool* bad)
{
    const int id = a.ids[t];
    if (id < 0) return 0;
    int s = -1;
    if (id < a.n_ids) s = a.id2slot[id];
    if (s >= 0 && s < a.n_slots) return s + 1;
    *bad = true;
    return 0;
}

__global__ __launch_bounds__(kBT) void bucket_runs_rows_kernel(BucketArgs a)
{
    __shared__ int s_wave[kNW + 1];
    __shared__ int s_key[kBT];
    static_assert(kBT % kPieceRows == 0, "pieces must not span chunks");
    const int tid = threadIdx.x, c = blockIdx.x;
    const int t = c * kBT + tid;
    const bool valid = t < a.T;
    bool bad = false;
    const int key = valid ? runs_key(a, t, &bad) : 0;
    bool prev_bad = false;                                   // reported by the chunk that owns that token
    const int first_prev = (tid == 0 && c > 0) ? runs_key(a, t - 1, &prev_bad) : 0;
    s_key[tid] = key;
    if (bad) atomicOr(a.flags, 1u);
    __syncthreads();
    int seg_head = 0, piece_head = 0;
    if (valid) {
        const int s = key - 1;
        a.perm[t] = t;
        a.row_slot[t] = s;
        a.row_rank[t] = s >= 0 ? a.slot_rank[s] : 0;
        a.row_loc[t] = s >= 0 ? a.slot_loc[s] : -1;
        a.row_scale[t] = s >= 0 ? a.slot_scale[s] : 0.f;
        const int prev = tid > 0 ? s_key[tid - 1] : first_prev;
        seg_head = (t == 0) || prev != key;
        piece_head = seg_head || (t % kPieceRows) == 0;
    }
    int n_seg, n_piece;
    block_excl_scan(seg_head, s_wave, &n_seg);
    block_excl_scan(piece_head, s_wave, &n_piece);
    if (tid == 0) {
        a.tok_key[2 * c] = n_seg;
        a.tok_key[2 * c + 1] = n_piece;
    }
}

__global__ __launch_bounds__(kBT) void bucket_runs_number_kernel(BucketArgs a)
{
    __shared__ int s_wave[kNW + 1];
    __shared__ int s_slot[kBT + 1];                          // [0]: the token in front of the chunk
    __shared__ int s_pstart[kBT + 1];
    const int tid = threadIdx.x, c = blockIdx.x, n_chunks = gridDim.x;
    const int t = c * kBT + tid;
    const int T = a.T;
    const bool valid = t < T;
    const int chunk_end = (c + 1) * kBT < T ? (c + 1) * kBT : T;
    // heads in the chunks in front of this one
    int seg_before = 0, piece_before = 0;
    for (int k = tid; k < c; k += kBT) {
        seg_before += a.tok_key[2 * k];
        piece_before += a.tok_key[2 * k + 1];
    }
    int seg_base, piece_base;
    block_excl_scan(seg_before, s_wave, &seg_base);
    block_excl_scan(piece_before, s_wave, &piece_base);
    const int s = valid ? a.row_slot[t] : -2;
    s_slot[tid + 1] = s;
    if (tid == 0) s_slot[0] = c > 0 ? a.row_slot[t - 1] : -2;
    __syncthreads();
    int seg_head = 0, piece_head = 0;
    if (valid) {
        seg_head = (t == 0) || s_slot[tid] != s;
        piece_head = seg_head || (t % kPieceRows) == 0;
    }
    int n_seg, n_piece;
    const int seg_ex = block_excl_scan(seg_head, s_wave, &n_seg);
    const int piece_ex = block_excl_scan(piece_head, s_wave, &n_piece);
    if (seg_head) {
        a.seg_start[seg_base + seg_ex] = t;
        a.seg_slot[seg_base + seg_ex] = s;
    }
    if (piece_head) s_pstart[piece_ex] = t;
    if (tid == 0) s_pstart[n_piece] = chunk_end;
    __syncthreads();
    if (piece_head) {
        const int p = piece_base + piece_ex;
        a.piece_start[p] = t;
        a.piece_slot[p] = s;
        int4 rec;
        rec.x = t;
        rec.y = s_pstart[piece_ex + 1] - t;
        rec.z = s >= 0 ? a.slot_loc[s] : -1;
        rec.w = s >= 0 ? a.slot_rank[s] : 0;
        reinterpret_cast<int4*>(a.piece_info)[p] = rec;
    }
    if (c == n_chunks - 1 && tid == 0) {
        a.seg_start[seg_base + n_seg] = T;
        a.piece_start[piece_base + n_piece] = T;
        *a.n_seg = seg_base + n_seg;
        *a.n_pieces = piece_base + n_piece;
    }
}

__global__ void meta_update_kernel(MetaUpdates u, int32_t* slot_rank, float* slot_scale, int32_t* slot_loc, int32_t* id2slot)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    for (int i = 0; i < u.n; ++i) {
        if (u.evicted[i] >= 0) id2slot[u.evicted[i]] = -1;
        slot_rank[u.slot[i]] = u.rank[i];
        slot_scale[u.slot[i]] = u.scale[i];
        slot_loc[u.slot[i]] = u.loc[i];
        if (u.adapter[i] >= 0) id2slot[u.adapter[i]] = u.slot[i];
    }
}

// blockIdx.y: matrix of the batch; the workgroups of a row stride over its 16-byte units.  The sources are
// pinned host memory read over the host link: enough 16-byte loads in flight per lane to keep it busy.
constexpr int kCopyThreads = 256, kCopyBlocksPerMatrix = 16, kCopyUnroll = 4;
__global__ __launch_bounds__(kCopyThreads) void copy_batch_kernel(CopyBatch b)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const int m = blockIdx.y;
    const u32x4* src = static_cast<const u32x4*>(b.src[m]);
    u32x4* dst = static_cast<u32x4*>(b.dst[m]);
    const uint32_t n = b.bytes[m] / 16;
    const uint32_t stride = gridDim.x * kCopyThreads;
    for (uint32_t i0 = blockIdx.x * kCopyThreads + threadIdx.x; i0 < n; i0 += stride * kCopyUnroll) {
        u32x4 v[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (i0 + u * stride < n) v[u] = __builtin_nontemporal_load(src + i0 + u * stride);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (i0 + u * stride < n) dst[i0 + u * stride] = v[u];
    }
}

__global__ void fill_i32_kernel(int32_t* p, int32_t value, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = value;
}

}  // namespace

hipError_t launch_bucket(const BucketArgs& a, hipStream_t stream)
{
    if (a.mode != 0 && a.T > kFastT) {
        const int chunks = (a.T + kBT - 1) / kBT;
        hipLaunchKernelGGL(bucket_runs_rows_kernel, dim3(chunks), dim3(kBT), 0, stream, a);
        hipLaunchKernelGGL(bucket_runs_number_kernel, dim3(chunks), dim3(kBT), 0, stream, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(bucket_kernel, dim3(1), dim3(kBT), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_meta_update(const MetaUpdates& u, int32_t* slot_rank, float* slot_scale, int32_t* slot_loc,
                              int32_t* id2slot, hipStream_t stream)
{
    hipLaunchKernelGGL(meta_update_kernel, dim3(1), dim3(kWave), 0, stream, u, slot_rank, slot_scale, slot_loc, id2slot);
    return hipGetLastError();
}

hipError_t launch_copy_batch(const CopyBatch& b, hipStream_t stream)
{
    if (b.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_batch_kernel, dim3(kCopyBlocksPerMatrix, b.n), dim3(kCopyThreads), 0, stream, b);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, int32_t value, size_t n, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, value, n);
    return hipGetLastError();
}

}  // namespace lora
