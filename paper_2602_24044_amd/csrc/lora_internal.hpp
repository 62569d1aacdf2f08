// Internal declarations shared by the host code and the HIP kernels of liblora_mi355.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace lora {

constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kPieceRows = 32;       // grouped rows are cut into pieces that never cross a 32-row window
constexpr int kBK = 64;              // K extent of one LDS tile (bf16 elements)
constexpr int kMaxSlots = 4095;
constexpr int kMaxProj = 16;
constexpr int kMaxLayers = 256;
constexpr int kMaxRank = 64;
constexpr int kMetaBatch = 16;       // slot-metadata updates carried by one kernel launch
constexpr int kSplitMaxTokens = 1024;// largest T served by the split-K path
constexpr int kShrinkKC = 1024;      // K extent of one shrink work item on the split-K path
constexpr int kMaxShrinkChunks = 64;
constexpr int kLocUnit = 64;               // bf16 elements (128 bytes) per unit of an adapter's location in the slot region
constexpr int kPageRanks = 8;              // rank units per page of a paged slot region
constexpr uint32_t kFlagInternal = 2u;     // LORA_FLAG_INTERNAL: a bounded wait inside a kernel expired
constexpr int kShrinkWaitSpins = 400000;  // bounded wait of the tile workgroups for the launch's shrink workgroups (~1 us each)

// Device-side view of a context: everything the kernels need, passed by value.
struct DeviceView {
    // slot region
    const uint16_t* slots;     // bf16 bits: the slot region (uniform slots, or the pool of pages)
    const int32_t* slot_rank;  // [n_slots]
    const float* slot_scale;   // [n_slots]
    // segment map of the current step (grouped order)
    const int32_t* perm;       // [T]
    const int32_t* row_slot;   // [T] slot of each grouped position
    const int32_t* row_loc;    // [T] where that slot's adapter starts: kLocUnit-element units from `slots`; -1: none
    const int32_t* row_rank;   // [T] rank of that slot's adapter (0 for backbone-only rows)
    const float* row_scale;    // [T] scale of that slot's adapter
    const int32_t* piece_start;// [n_pieces + 1]
    const int32_t* piece_slot; // [n_pieces]
    const int32_t* n_pieces;   // [1]
    const int32_t* piece_info; // [n_pieces][4]: first grouped row, rows, location of the adapter (as row_loc), rank (one 16-byte load)
    int32_t T;
    int32_t max_rank;
};

struct BucketArgs {
    const int32_t* ids;
    int32_t T;
    int32_t mode;
    const int32_t* id2slot;
    int32_t n_ids;
    int32_t n_slots;
    int32_t* perm;
    int32_t* row_slot;
    int32_t* row_loc;
    const int32_t* slot_loc;   // [n_slots] location of the adapter in each slot (see DeviceView::row_loc)
    int32_t* row_rank;
    float* row_scale;
    const int32_t* slot_rank;
    const float* slot_scale;
    int32_t* seg_start;
    int32_t* seg_slot;
    int32_t* n_seg;
    int32_t* piece_start;
    int32_t* piece_slot;
    int32_t* n_pieces;
    int32_t* piece_info;
    int32_t* tok_key;
    uint32_t* flags;
};

struct MetaUpdates {
    int32_t n;
    int32_t slot[kMetaBatch];
    int32_t adapter[kMetaBatch];   // adapter now in the slot (or -1)
    int32_t evicted[kMetaBatch];   // adapter that left the slot (or -1)
    int32_t rank[kMetaBatch];
    int32_t loc[kMetaBatch];       // where the adapter's weights start (DeviceView::row_loc units), -1: none
    float scale[kMetaBatch];
};

// Adapter matrices on their way from pinned host memory into their slots: one launch copies a batch of them,
// reading the host memory directly (paper Sec. 2.2: adapters are swapped in from CPU memory).
constexpr int kCopyBatch = 32;
struct CopyBatch {
    int32_t n;
    int32_t pad_;
    const void* src[kCopyBatch];   // device-visible address of pinned host memory
    void* dst[kCopyBatch];         // inside a slot
    uint32_t bytes[kCopyBatch];    // multiple of 16
};

// One launch can serve several projections that share d_in ("packed projections": q|k|v, gate|up), each with
// its own x, W, out and adapter matrices.  The slices sit side by side along N: tiles, 32-column blocks of the
// split-K partial matrix and shrink work items are numbered across them.
constexpr int kMaxGroup = 4;
struct Slice {
    const uint16_t* x;   // [T, K] bf16
    const uint16_t* W;   // [N, K] bf16
    uint16_t* out;       // [T, N] bf16
    float* vpart;        // [n_kc][T][max_rank] fp32: this slice's shrink results
    size_t a_unit;       // elements in front of this projection's A and B inside a slot, per unit of the rank of
    size_t b_unit;       // the adapter in it (the adapter is stored packed at its own rank)
    int32_t N;
    int32_t tile0;       // first N tile of the slice (set by the GEMM launcher for its tile width)
    int32_t blk0;        // first 32-column block of the slice in the packed partial matrix (multiple of 4)
    int32_t pad_;
    const uint16_t* bias;// [N] bf16 bias of the backbone layer, or null
};
struct GroupArgs {
    int32_t n;
    int32_t pad_;
    Slice s[kMaxGroup];
};

struct ShrinkArgs {
    DeviceView dv;
    GroupArgs g;         // x, a_unit and vpart of every slice
    int32_t K;
    int32_t n_kc;        // K chunks (one partial result each)
    int32_t kc_len;      // K extent of a chunk (multiple of 64); the waves of a workgroup share a chunk
    int32_t on;          // 0: nothing to shrink (no adapter resident)
};

struct GemmArgs {
    DeviceView dv;
    GroupArgs g;
    int32_t K;
    int32_t tiles_m, tiles_n;   // tiles_n counts the tiles of all slices
    int32_t split_k;     // 1 on the fused path
    int32_t n_kc;
    int32_t nblk;        // 32-column blocks per row block of the packed partial matrix
    float* part;         // split path: [split_k][Mpad / 32][nblk][1024] fp32, row blocks counted from m_begin
    int32_t Mpad;
    int32_t m_begin, m_end;     // grouped rows served by this launch (m_begin a multiple of 256); tiles start at m_begin
    // split path of the 64-wide-K kernels: workgroups main_grid .. grid - 1 only do shrink items, shrink_q each,
    // while the tile workgroups stream; what is left is shared out over every workgroup (0: every workgroup
    // takes the items blockIdx, blockIdx + grid, ... after its tile)
    int32_t main_grid;
    int32_t shrink_q;
    // fused path of the 64-wide-K kernels: the first shrink_front workgroups of the grid do the launch's shrink
    // items (the tiles leave that many CUs idle) and the tile workgroups wait for them before their epilogue.
    // sync[0]: shrink workgroups that have finished, sync[1]: tile workgroups past the wait; the last of those
    // sets both back to zero.  The wait is bounded: when it expires, LORA_FLAG_INTERNAL is set in *flags.
    int32_t shrink_front;
    int32_t front_expect;       // reports the tile workgroups wait for: shrink_front (one more in the host-forced test of the expired wait)
    int32_t wait_spins;         // polls of the bounded wait
    int32_t pad_;
    uint32_t* sync;
    uint32_t* flags;
};

struct ReduceArgs {
    DeviceView dv;
    GroupArgs g;
    int32_t split_k;
    int32_t Mpad;
    int32_t nblk;
    const float* part;
    int32_t n_kc;
    int32_t m_begin, m_end;     // grouped rows served by this launch (as in the split-K GEMM before it)
};

// launchers (defined next to their kernels); every launch is asynchronous on `stream`
hipError_t launch_bucket(const BucketArgs& a, hipStream_t stream);
hipError_t launch_meta_update(const MetaUpdates& u, int32_t* slot_rank, float* slot_scale, int32_t* slot_loc,
                              int32_t* id2slot, hipStream_t stream);
hipError_t launch_fill_i32(int32_t* p, int32_t value, size_t n, hipStream_t stream);
hipError_t launch_copy_batch(const CopyBatch& b, hipStream_t stream);
hipError_t launch_shrink(const ShrinkArgs& a, int grid, hipStream_t stream);
hipError_t launch_gemm_fused(const GemmArgs& a, int variant, hipStream_t stream, const char** name);
hipError_t launch_gemm_splitk(const GemmArgs& a, const ShrinkArgs& sa, int variant, hipStream_t stream, const char** name);
// K walked in 64-wide tiles (whole 128-byte lines per row segment): the small-batch kernels
hipError_t launch_gemm_rows128_fused(const GemmArgs& a, const ShrinkArgs& sa, int variant, hipStream_t stream, const char** name);
hipError_t launch_gemm_rows128_splitk(const GemmArgs& a, const ShrinkArgs& sa, int variant, hipStream_t stream, const char** name);
// large batches: tiles staged through registers (ordinary loads + LDS writes)
hipError_t launch_gemm_rows128_glu(const GemmArgs& a, const ShrinkArgs& none, int variant, hipStream_t stream,
                                   const char** name);
hipError_t launch_gemm_staged_glu(const GemmArgs& a, hipStream_t stream, const char** name);
hipError_t launch_gemm_staged_fused(const GemmArgs& a, int variant, hipStream_t stream, const char** name);
hipError_t launch_reduce_expand(const ReduceArgs& a, int grid, hipStream_t stream);

}  // namespace lora
