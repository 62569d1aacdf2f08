// Host side of liblora_mi355: context, slot table with least-recently-used replacement, and the
// launch sequences behind lora_slots_load / lora_bucket / lora_layer_forward.
#include "../../include/lora_mi355.h"
#include "lora_internal.hpp"

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace lora;

// Scratch of lora_layer_forward_static, for callers that may not allocate and hand in no workspace: split-K
// partial tiles first, the shrink results behind them.  Every GPU the library runs on holds its own copy of the
// array until the process ends.  In host code this name is only a handle for hipGetSymbolAddress: the kernels
// get the address that call returns (static_scratch_of), never the name itself.
constexpr size_t kStaticPartBytes = 32u << 20;
constexpr size_t kStaticVpartBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticPartBytes + kStaticVpartBytes];

namespace {

thread_local std::string g_last_hip_error;

inline bool hip_fail(hipError_t e, const char* what)
{
    if (e == hipSuccess) return false;
    g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    return true;
}
#define HIP_FAIL(call) hip_fail((call), #call)

// Device address of `scratch` on the current device, looked up once per device (with that device current).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

bool static_scratch_of(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices) return false;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        if (HIP_FAIL(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return false;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return true;
}

constexpr size_t kAlign = 256;
constexpr size_t kEngineRunBytes = 128u << 10; // shortest run for which a copy call per run pays
constexpr int kMarkedCallsPerLoad = 64;        // calls after a load that still mark their end for the next load (see lora_ctx)
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
    size_t slot_stride_elems = 0;          // bf16 elements per slot (uniform slots)
    size_t page_stride_elems = 0;          // bf16 elements per page of kPageRanks rank units (paged slots)
    // An adapter sits in its slot packed at its own rank r: layer after layer, per layer the A [r, d_in] and
    // B [d_out, r] of every projection back to back.  a_unit / b_unit [n_layers * n_proj]: elements in front of
    // that matrix per unit of rank (its offset inside the slot is r times that), so one adapter is one run of
    // r * unit_total elements at the start of its slot, whatever its rank.
    std::vector<size_t> a_unit, b_unit;
    size_t unit_total = 0;
    size_t off_slots = 0, off_slot_rank = 0, off_slot_scale = 0, off_id2slot = 0, off_header = 0;
    size_t off_row_rank = 0, off_row_scale = 0, off_row_loc = 0, off_slot_loc = 0;
    size_t off_perm = 0, off_row_slot = 0, off_seg_start = 0, off_seg_slot = 0, off_piece_start = 0,
           off_piece_slot = 0, off_piece_info = 0, off_tok_key = 0, off_vpart = 0, off_part = 0;
    size_t vpart_elems = 0, part_elems = 0;
    size_t total = 0;
};

// split-K GEMM variants 3, 4 and 7 use 128-row tiles, the others 256-row tiles; 6 and 7 walk K in 64-wide tiles
int split_bm(int variant) { return (variant == 3 || variant == 4 || variant == 7) ? 128 : 256; }

// Device-visible address of a pointer into pinned (page-locked, mapped) host memory, or NULL when the pointer
// is anything else (pageable host memory must never reach a kernel).
const void* device_view_of_pinned(const void* p)
{
    hipPointerAttribute_t at;
    std::memset(&at, 0, sizeof at);
    if (hipPointerGetAttributes(&at, p) != hipSuccess) {
        (void)hipGetLastError();      // an unknown (pageable) pointer is reported as an error: clear it
        return nullptr;
    }
    if (at.type != hipMemoryTypeHost || !at.devicePointer) return nullptr;
    return at.devicePointer;
}

// Compute units of the current device (256 on an MI355X); 256 when there is no device to ask.
int device_cus()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        n < 8) {
        (void)hipGetLastError();
        return 256;
    }
    return n;
}

int auto_split_cap(int N, int n_cus)
{
    const int tiles_n = (N + 127) / 128;
    int s = (n_cus + tiles_n - 1) / tiles_n;
    return std::max(1, std::min(16, s));
}

// Tile shape of the fused GEMM: rounds of workgroups over the CUs times the cost of one tile, with the
// per-flop efficiencies measured for the three shapes (256x256: 1, 256x128: 0.78, 128x128: 0.65).  Large
// problems take the big tile; a projection with few big tiles (k/v at a few thousand tokens) fills the chip
// better with small ones.
template <typename TilesOf>
int pick_fused_variant(int n_cus, TilesOf&& tiles_of)
{
    auto rounds = [&](int bm, int bn) { return (double)((tiles_of(bm, bn) + n_cus - 1) / n_cus); };
    const double big = rounds(256, 256) * 1.0, mid = rounds(256, 128) * (0.5 / 0.78), small = rounds(128, 128) * (0.25 / 0.65);
    if (big <= mid * 1.1 && big <= small * 1.1) return 0;      // near ties go to the big tile (measured)
    return mid <= small ? 4 : 3;
}

bool valid_config(const lora_config* c)
{
    if (!c || !c->proj) return false;
    if (c->n_slots < 1 || c->n_slots > kMaxSlots) return false;
    if (c->max_rank < 8 || c->max_rank > kMaxRank || c->max_rank % 8) return false;
    if (c->n_proj < 1 || c->n_proj > kMaxProj) return false;
    if (c->n_layers < 0 || c->n_layers > kMaxLayers) return false;
    if (c->max_tokens < 1 || c->max_adapter_id < 0) return false;
    if (c->path < LORA_PATH_AUTO || c->path > LORA_PATH_SPLITK) return false;
    if (c->split_k < 0 || c->split_k > 16) return false;
    if (c->n_pages < 0 || (c->n_pages > 0 && c->n_pages < c->max_rank / kPageRanks)) return false;
    {
        // an adapter's place in the slot region is a 32-bit count of 128-byte units
        uint64_t unit = 0;
        for (int p = 0; p < c->n_proj; ++p) unit += (uint64_t)std::max(0, c->proj[p].d_in) + (uint64_t)std::max(0, c->proj[p].d_out);
        unit *= (uint64_t)std::max(1, c->n_layers);
        const uint64_t region = c->n_pages > 0 ? (unit * kPageRanks + kLocUnit) * (uint64_t)c->n_pages
                                               : (unit * (uint64_t)c->max_rank + 2 * kLocUnit) * (uint64_t)c->n_slots;
        if (region / kLocUnit >= (1ull << 31)) return false;
    }
    for (int p = 0; p < c->n_proj; ++p) {
        if (c->proj[p].d_in < 64 || c->proj[p].d_in % 64) return false;
        if (c->proj[p].d_out < 8 || c->proj[p].d_out % 8) return false;
        // tile copies address x and W with 32-bit element offsets
        if ((uint64_t)c->max_tokens * (uint64_t)c->proj[p].d_in >= (1ull << 32)) return false;
        if ((uint64_t)c->proj[p].d_out * (uint64_t)c->proj[p].d_in >= (1ull << 32)) return false;
    }
    return true;
}

Layout make_layout(const lora_config* c, int n_cus)
{
    Layout L;
    size_t e = 0;
    int k_max = 0;
    const int n_layers = std::max(1, c->n_layers);
    L.a_unit.resize((size_t)n_layers * c->n_proj);
    L.b_unit.resize((size_t)n_layers * c->n_proj);
    for (int l = 0; l < n_layers; ++l)
        for (int p = 0; p < c->n_proj; ++p) {
            const size_t f = (size_t)l * c->n_proj + p;
            L.a_unit[f] = e;
            e += (size_t)c->proj[p].d_in;
            L.b_unit[f] = e;
            e += (size_t)c->proj[p].d_out;
            k_max = std::max(k_max, c->proj[p].d_in);
        }
    L.unit_total = e;
    L.slot_stride_elems = align_up(e * (size_t)c->max_rank * 2, kAlign) / 2;
    L.page_stride_elems = align_up(e * (size_t)kPageRanks * 2, (size_t)kLocUnit * 2) / 2;
    const size_t Tm = (size_t)c->max_tokens;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, kAlign); return at; };
    L.off_slots = c->n_pages > 0 ? take(L.page_stride_elems * 2 * (size_t)c->n_pages)
                                 : take(L.slot_stride_elems * 2 * (size_t)c->n_slots);
    L.off_slot_rank = take(4 * (size_t)c->n_slots);
    L.off_slot_loc = take(4 * (size_t)c->n_slots);
    L.off_slot_scale = take(4 * (size_t)c->n_slots);
    L.off_id2slot = take(4 * ((size_t)c->max_adapter_id + 1));
    L.off_header = take(256);
    L.off_perm = take(4 * Tm);
    L.off_row_slot = take(4 * Tm);
    L.off_row_rank = take(4 * Tm);
    L.off_row_scale = take(4 * Tm);
    L.off_row_loc = take(4 * Tm);
    L.off_seg_start = take(4 * (Tm + 1));
    L.off_seg_slot = take(4 * Tm);
    const size_t max_pieces = Tm + Tm / kPieceRows + 2;
    L.off_piece_start = take(4 * (max_pieces + 1));
    L.off_piece_slot = take(4 * max_pieces);
    L.off_piece_info = take(16 * max_pieces);
    L.off_tok_key = take(4 * Tm);
    const size_t Ts = std::min<size_t>(Tm, kSplitMaxTokens);
    const size_t kc_max = std::min<size_t>(kMaxShrinkChunks, ((size_t)k_max + kShrinkKC - 1) / kShrinkKC);
    L.vpart_elems = kMaxGroup * std::max(Tm * (size_t)c->max_rank, Ts * (size_t)c->max_rank * kc_max);
    L.off_vpart = take(4 * L.vpart_elems);
    size_t part_cols = 0;
    for (int p = 0; p < c->n_proj; ++p) {
        const int s = c->split_k > 0 ? c->split_k : auto_split_cap(c->proj[p].d_out, n_cus);
        part_cols = std::max(part_cols, align_up((size_t)c->proj[p].d_out, 32) * (size_t)s);
    }
    L.part_elems = align_up(Ts, 256) * part_cols;
    L.off_part = take(4 * L.part_elems);
    L.total = o;
    return L;
}

struct ProfileSlot {
    hipEvent_t beg, end;
    const char* name;
};

}  // namespace

struct lora_ctx {
    lora_config cfg;
    std::vector<lora_proj_shape> proj;
    Layout L;
    bool host_only = false;
    char* base = nullptr;
    int device = -1;                        // the device the context was created on
    int n_cus = 256;                        // its compute units: what a launch can keep busy at once
    char* static_scratch = nullptr;         // that device's copy of `scratch` (lora_layer_forward_static)

    // host slot table
    std::vector<int32_t> slot_adapter, slot_rank_h;
    std::vector<float> slot_scale_h;
    std::vector<uint64_t> slot_last_used;
    std::vector<int32_t> id2slot_h;
    // paged slots (cfg.n_pages > 0): first page of every slot's adapter (-1: none) and the slot that holds each page
    std::vector<int32_t> slot_first_page, page_owner;
    uint64_t tick = 0;
    int n_resident = 0;

    // stream ordering
    hipEvent_t ev_meta = nullptr, ev_fwd = nullptr;
    // copies are enqueued in units (a projection; a whole layer when there are several layers), one event each
    std::vector<hipEvent_t> ev_unit;
    bool meta_pending = false;
    std::vector<char> unit_pending;
    int n_layers = 1;
    int unit_of(int layer, int proj) const { return n_layers > 1 ? layer : proj; }
    hipStream_t copy_stream = nullptr;      // stream of the latest load
    hipStream_t last_fwd_stream = nullptr;
    bool have_fwd = false;
    // A context that loads adapters between its steps marks the end of each of its calls with ev_fwd (fwd_marked:
    // ev_fwd stands behind the last call), so that a load waits for this context's work only; the calls after
    // which that is still done are counted down from every load.  Without the mark a load records the event at
    // the tail of the stream and so also waits for what other contexts have enqueued there since.
    bool fwd_marked = false;
    int marks_left = 0;
    bool work_enqueued(hipStream_t s)
    {
        last_fwd_stream = s;
        have_fwd = true;
        fwd_marked = false;
        if (marks_left > 0) {
            --marks_left;
            if (hipEventRecord(ev_fwd, s) != hipSuccess) return false;
            fwd_marked = true;
        }
        return true;
    }

    int32_t tune[8] = {0};
    bool inline_shrink_off = false;         // a bounded wait inside a launch has expired once: shrink as a launch of its own from then on
    std::vector<const uint16_t*> bias;      // [n_layers * n_proj] device, caller-owned (lora_set_bias)

    // current segment map
    uint64_t epoch = 0;
    int32_t seg_T = -1, seg_mode = 0;

    // launch log / profiling
    std::vector<const char*> last_launches;
    bool profiling = false;
    std::vector<ProfileSlot> prof_pool;
    size_t prof_used = 0;
    std::vector<std::string> prof_names;
    std::vector<double> prof_ms;
    std::vector<int64_t> prof_count;

    template <typename Tp> Tp* dev(size_t off) const { return reinterpret_cast<Tp*>(base + off); }
    int32_t* d_slot_rank() const { return dev<int32_t>(L.off_slot_rank); }
    int32_t* d_slot_loc() const { return dev<int32_t>(L.off_slot_loc); }
    // where the adapter of a slot starts, in kLocUnit-element units from the start of the slot region
    int32_t loc_of(int slot, int first_page) const
    {
        if (cfg.n_pages > 0) return first_page < 0 ? -1 : (int32_t)((size_t)first_page * L.page_stride_elems / kLocUnit);
        return (int32_t)((size_t)slot * L.slot_stride_elems / kLocUnit);
    }
    float* d_slot_scale() const { return dev<float>(L.off_slot_scale); }
    int32_t* d_id2slot() const { return dev<int32_t>(L.off_id2slot); }
    uint32_t* d_flags() const { return dev<uint32_t>(L.off_header); }
    int32_t* d_n_seg() const { return dev<int32_t>(L.off_header) + 1; }
    int32_t* d_n_pieces() const { return dev<int32_t>(L.off_header) + 2; }

    DeviceView view(int32_t T) const
    {
        DeviceView v;
        v.slots = dev<uint16_t>(L.off_slots);
        v.slot_rank = d_slot_rank();
        v.slot_scale = d_slot_scale();
        v.perm = dev<int32_t>(L.off_perm);
        v.row_slot = dev<int32_t>(L.off_row_slot);
        v.row_loc = dev<int32_t>(L.off_row_loc);
        v.row_rank = dev<int32_t>(L.off_row_rank);
        v.row_scale = dev<float>(L.off_row_scale);
        v.piece_start = dev<int32_t>(L.off_piece_start);
        v.piece_slot = dev<int32_t>(L.off_piece_slot);
        v.n_pieces = d_n_pieces();
        v.piece_info = dev<int32_t>(L.off_piece_info);
        v.T = T;
        v.max_rank = cfg.max_rank;
        return v;
    }
};

namespace {

// Brackets one kernel launch with timing events while profiling is on.
struct LaunchScope {
    lora_ctx* c;
    hipStream_t s;
    ProfileSlot* slot = nullptr;
    LaunchScope(lora_ctx* ctx, hipStream_t stream, const char* name) : c(ctx), s(stream)
    {
        c->last_launches.push_back(name);
        if (c->profiling && c->prof_used < c->prof_pool.size()) {
            slot = &c->prof_pool[c->prof_used++];
            slot->name = name;
            (void)hipEventRecord(slot->beg, s);
        }
    }
    void rename(const char* name)
    {
        c->last_launches.back() = name;
        if (slot) slot->name = name;
    }
    ~LaunchScope()
    {
        if (slot) (void)hipEventRecord(slot->end, s);
    }
};

// What one forward call (a projection or a packed group over T tokens) launches: path, tile variant, K split and
// the K chunks of the shrink.  Host arithmetic only.
struct ForwardPlan {
    int K = 0, Mpad = 0, n_max = 0;
    long n_pad_total = 0;       // columns of all slices, each padded to a multiple of 128
    bool split = false;         // split-K GEMM + reduce; otherwise shrink + fused GEMM
    bool dyn_shrink = false;    // split path: a share of the workgroups only shrinks
    int S = 1;                  // K split
    int split_variant = 0;
    int n_kc = 1, kc_len = 0;   // K chunks of the shrink and their length
};

lora_status plan_forward(const lora_ctx* c, int32_t T, int32_t n, const int32_t* projs, size_t part_elems,
                         size_t vpart_elems, ForwardPlan& out, bool fused_only = false)
{
    const int K = c->proj[projs[0]].d_in;
    // the slices sit side by side along N, each padded to a multiple of 128 columns
    long n_pad_total = 0;
    int n_max = 0;
    for (int k = 0; k < n; ++k) {
        n_pad_total += (long)align_up((size_t)c->proj[projs[k]].d_out, 128);
        n_max = std::max(n_max, c->proj[projs[k]].d_out);
    }
    auto tiles_of = [&](int bm, int bn) {
        long t = 0;
        for (int k = 0; k < n; ++k) t += (c->proj[projs[k]].d_out + bn - 1) / bn;
        return t * ((T + bm - 1) / bm);
    };

    // ---- plan ----
    const int Mpad = (T + 255) / 256 * 256;
    bool split = false, dyn_shrink = false;
    int S = 1;
    int split_variant = c->tune[LORA_TUNE_SPLIT_VARIANT];
    if (T <= kSplitMaxTokens) {
        if (c->cfg.path == LORA_PATH_SPLITK) split = true;
        else if (c->cfg.path == LORA_PATH_AUTO) split = tiles_of(256, 256) < c->n_cus / 2;
    }
    if (fused_only) split = false;
    if (split) {
        // narrow launches (k, v alone) fill the chip better with square 128 x 128 tiles
        // small batches walk K in 64-wide tiles (whole cache lines per row segment).  Narrow launches (k, v
        // alone) fill the chip better with square 128 x 128 tiles, and so does a 4096-wide projection over a
        // short K at up to 256 tokens (half the K splits, half the partial tiles)
        // and up to 128 tokens a 256-row tile would copy and multiply rows that do not exist
        if (split_variant == 0)
            split_variant = (T <= 128 || n_pad_total <= 2048 || (n_pad_total <= 4096 && K <= 8192 && T <= 256)) ? 7 : 6;
        const int bm = split_bm(split_variant), bn = split_variant == 2 ? 64 : 128;
        const long tiles = tiles_of(bm, bn);
        // The 64-wide-K kernels give a quarter of the CUs workgroups that only shrink, from the start (a shrink
        // item is a chain of dependent loads: behind the tile it would be a tail that no other work hides).
        // Only while those workgroups can finish the items meanwhile: a batch spread over hundreds of adapters
        // has more shrink work than tile work, and every workgroup takes its share after its tile instead.
        const long pieces_bound = (long)n * std::min<long>(T, (long)c->n_resident + (T + kPieceRows - 1) / kPieceRows);
        dyn_shrink = c->n_resident > 0 && (split_variant == 6 || split_variant == 7 || split_variant == 9) &&
                     pieces_bound * std::max(1, K / 2048) <= 512;
        const long target = dyn_shrink ? c->n_cus * 3 / 4 : c->n_cus;
        // K splits, at most 8, by a cost model in microseconds: a workgroup walking all of K moves (bm + bn) K
        // bf16 through its CU at about 48 GB/s, a launch takes ceil(tiles S / target) rounds of 1 / S of that
        // (one workgroup per CU: a grid just above the CU count costs a whole extra round), and every split
        // writes and reads back a set of fp32 partial tiles at about 5 TB/s.
        if (c->cfg.split_k > 0) {
            S = c->cfg.split_k;
        } else {
            const double t_full = (double)(bm + bn) * K * 2.0 / 48e3;
            const double t_part = (double)Mpad * (double)n_pad_total * 8.0 / 5e6;
            double best = 0.0;
            for (int cand = 1; cand <= 8; ++cand) {
                // a single K range takes the fused path instead (below): every CU can hold a tile and there are
                // no partial tiles at all
                const bool fused_instead = cand == 1 && c->cfg.path == LORA_PATH_AUTO;
                const long per_round = fused_instead ? c->n_cus : target;
                const double rounds = (double)((tiles * cand + per_round - 1) / per_round);
                double t_tiles = t_full * rounds / cand;
                if (dyn_shrink && !fused_instead) {
                    // the workgroups that only shrink run beside the tiles and the launch ends with the later of
                    // the two: about 7 us until a workgroup's first item is under way, then 5 us per item (a
                    // piece over 2048 of K); fewer splits leave more CUs to them
                    const long shrinkers = std::max<long>(1, std::min<long>(c->n_cus / 2, c->n_cus - tiles * cand));
                    const double items = (double)pieces_bound * std::max(1, K / 2048);
                    t_tiles = std::max(t_tiles, 7.0 + 5.0 * items / (double)shrinkers);
                }
                const double cost = t_tiles + (fused_instead ? 0.0 : t_part * cand);
                if (cand == 1 || cost < best) {
                    best = cost;
                    S = cand;
                }
            }
        }
        S = std::min(S, std::max(1, (K / kBK) / 2));
        const size_t cap = part_elems / ((size_t)Mpad * (size_t)n_pad_total);
        S = (int)std::min<size_t>((size_t)S, std::max<size_t>(cap, 1));
        if ((size_t)S * Mpad * (size_t)n_pad_total > part_elems) return LORA_ERR_OOM;
        // a single K range would only add the round trip of the partial tiles: the launch already fills
        // the chip, take the fused path with the same tile
        if (S == 1 && c->cfg.path == LORA_PATH_AUTO) split = false;
        if (!split) dyn_shrink = false;
    }
    int n_kc = 1, kc_len = K;
    if (T <= kSplitMaxTokens) {
        n_kc = std::min<int>(kMaxShrinkChunks, (K + kShrinkKC - 1) / kShrinkKC);
        if (split && dyn_shrink) {
            // chunks of 2048: one round of operand loads per wavefront and item
            n_kc = std::max(1, std::min<int>(kMaxShrinkChunks, K / 2048));
        } else if (split) {
            // The shrink items (slice x piece x K chunk) are shared out over the workgroups of the split GEMM,
            // each item a dependent load -> MFMA -> reduce chain: no more chunks than give every workgroup
            // one item (when there are more pieces than workgroups, fine chunks balance better and stay).
            // The piece count is only known on the device; this is its upper bound.
            const int bm = split_bm(split_variant), bn = split_variant == 2 ? 64 : 128;
            const long wgs = tiles_of(bm, bn) * S;
            const long pieces = (long)n * std::min<long>(T, (long)c->n_resident + (T + kPieceRows - 1) / kPieceRows);
            if (pieces <= wgs) n_kc = (int)std::max<long>(1, std::min<long>(n_kc, wgs / std::max<long>(pieces, 1)));
        }
        kc_len = ((K + n_kc - 1) / n_kc + kBK - 1) / kBK * kBK;
        n_kc = (K + kc_len - 1) / kc_len;
    } else {
        // Larger batches run the shrink as a launch of its own, one item (piece x K chunk) per workgroup, two
        // workgroups per CU at a time.  A mixed step of a few thousand tokens has only a few hundred pieces, each a
        // chain of loads over all of K: K is cut until the launch has about four rounds of items (chunks of at least
        // 1024, as many as the scratch for the partial results holds).
        const long pieces = (long)n * ((T + kPieceRows - 1) / kPieceRows + std::min<long>(T, (long)c->n_resident));
        const long want = (8L * c->n_cus + pieces - 1) / std::max<long>(pieces, 1);
        const long room = (long)(vpart_elems / ((size_t)n * (size_t)T * (size_t)c->cfg.max_rank));
        n_kc = (int)std::max<long>(1, std::min<long>({want, (long)(K / kShrinkKC), room, (long)kMaxShrinkChunks}));
        kc_len = ((K + n_kc - 1) / n_kc + kBK - 1) / kBK * kBK;
        n_kc = (K + kc_len - 1) / kc_len;
    }
    out.K = K;
    out.Mpad = Mpad;
    out.n_max = n_max;
    out.n_pad_total = n_pad_total;
    out.split = split;
    out.dyn_shrink = dyn_shrink;
    out.S = S;
    out.split_variant = split_variant;
    out.n_kc = n_kc;
    out.kc_len = kc_len;
    return LORA_OK;
}

}  // namespace

extern "C" {

const char* lora_last_hip_error(void) { return g_last_hip_error.c_str(); }

const char* lora_status_string(lora_status status)
{
    // a C caller may hand in any integer: read the bits, not the enumeration (a value outside its range is not
    // one a C++ enumeration may hold)
    int s;
    std::memcpy(&s, &status, sizeof s);
    static_assert(sizeof(int) == sizeof(lora_status), "lora_status is passed as an int");
    switch (s) {
        case LORA_OK: return "ok";
        case LORA_ERR_INVALID_ARG: return "invalid argument";
        case LORA_ERR_SHAPE: return "unsupported shape or rank";
        case LORA_ERR_OOM: return "slab too small";
        case LORA_ERR_SLOT_RANGE: return "slot index out of range";
        case LORA_ERR_RANK_EXCEEDS_SMAX: return "adapter rank exceeds max_rank";
        case LORA_ERR_SLOTS_EXHAUSTED: return "no evictable slot";
        case LORA_ERR_NOT_RESIDENT: return "token names a non-resident adapter";
        case LORA_ERR_HIP: return "HIP runtime error";
        case LORA_ERR_ID_RANGE: return "adapter id out of range";
        case LORA_ERR_STARVATION: return "no starvation-free placement";
        case LORA_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

size_t lora_slab_bytes(const lora_config* cfg)
{
    if (!valid_config(cfg)) return 0;
    if (cfg->flags & LORA_CREATE_HOST_ONLY) return 0;
    return make_layout(cfg, device_cus()).total;
}

lora_status lora_create(const lora_config* cfg, lora_ctx** out)
{
    if (!out) return LORA_ERR_INVALID_ARG;
    *out = nullptr;
    if (!cfg || !cfg->proj) return LORA_ERR_INVALID_ARG;
    if (!valid_config(cfg)) {
        if (cfg->n_proj >= 1 && cfg->n_proj <= kMaxProj && cfg->n_slots >= 1 && cfg->max_tokens >= 1 &&
            cfg->max_adapter_id >= 0)
            return LORA_ERR_SHAPE;
        return LORA_ERR_INVALID_ARG;
    }
    lora_ctx* c = new (std::nothrow) lora_ctx();
    if (!c) return LORA_ERR_OOM;
    c->cfg = *cfg;
    c->proj.assign(cfg->proj, cfg->proj + cfg->n_proj);
    c->cfg.proj = c->proj.data();
    c->host_only = (cfg->flags & LORA_CREATE_HOST_ONLY) != 0;
    c->n_cus = c->host_only ? 256 : device_cus();
    c->L = make_layout(&c->cfg, c->n_cus);
    c->n_layers = std::max(1, cfg->n_layers);
    const size_t n_flat = (size_t)c->n_layers * cfg->n_proj;
    const size_t n_units = c->n_layers > 1 ? (size_t)c->n_layers : (size_t)cfg->n_proj;
    c->ev_unit.assign(n_units, nullptr);
    c->unit_pending.assign(n_units, 0);
    c->bias.assign(n_flat, nullptr);
    c->slot_adapter.assign(cfg->n_slots, -1);
    c->slot_rank_h.assign(cfg->n_slots, 0);
    c->slot_scale_h.assign(cfg->n_slots, 0.f);
    c->slot_last_used.assign(cfg->n_slots, 0);
    c->id2slot_h.assign((size_t)cfg->max_adapter_id + 1, -1);
    c->slot_first_page.assign(cfg->n_slots, -1);
    c->page_owner.assign((size_t)std::max(0, cfg->n_pages), -1);

    if (!c->host_only) {
        if (!cfg->slab || (reinterpret_cast<uintptr_t>(cfg->slab) % kAlign) != 0) {
            delete c;
            return LORA_ERR_INVALID_ARG;
        }
        if (cfg->slab_bytes < c->L.total) {
            delete c;
            return LORA_ERR_OOM;
        }
        c->base = static_cast<char*>(cfg->slab);
        // this device's copy of the static scratch array (lora_layer_forward_static), looked up once per device
        void* sp = nullptr;
        if (HIP_FAIL(hipGetDevice(&c->device)) || !static_scratch_of(c->device, &sp)) {
            delete c;
            return LORA_ERR_HIP;
        }
        c->static_scratch = static_cast<char*>(sp);
        bool ok = !HIP_FAIL(hipEventCreateWithFlags(&c->ev_meta, hipEventDisableTiming)) &&
                  !HIP_FAIL(hipEventCreateWithFlags(&c->ev_fwd, hipEventDisableTiming));
        for (size_t u = 0; ok && u < n_units; ++u)
            ok = !HIP_FAIL(hipEventCreateWithFlags(&c->ev_unit[u], hipEventDisableTiming));
        ok = ok && !HIP_FAIL(launch_fill_i32(c->d_slot_rank(), 0, cfg->n_slots, nullptr));
        ok = ok && !HIP_FAIL(launch_fill_i32(reinterpret_cast<int32_t*>(c->d_slot_scale()), 0, cfg->n_slots, nullptr));
        ok = ok && !HIP_FAIL(launch_fill_i32(c->d_id2slot(), -1, (size_t)cfg->max_adapter_id + 1, nullptr));
        ok = ok && !HIP_FAIL(launch_fill_i32(c->dev<int32_t>(c->L.off_header), 0, 64, nullptr));
        ok = ok && !HIP_FAIL(launch_fill_i32(c->dev<int32_t>(c->L.off_piece_start), 0, 1, nullptr));
        ok = ok && !HIP_FAIL(hipDeviceSynchronize());
        if (!ok) {
            (void)hipGetLastError();
            lora_destroy(c);
            return LORA_ERR_HIP;
        }
    }
    *out = c;
    return LORA_OK;
}

lora_status lora_destroy(lora_ctx* c)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    if (!c->host_only) {
        (void)hipDeviceSynchronize();
        if (c->ev_meta) (void)hipEventDestroy(c->ev_meta);
        if (c->ev_fwd) (void)hipEventDestroy(c->ev_fwd);
        for (hipEvent_t e : c->ev_unit)
            if (e) (void)hipEventDestroy(e);
        for (auto& s : c->prof_pool) {
            (void)hipEventDestroy(s.beg);
            (void)hipEventDestroy(s.end);
        }
    }
    delete c;
    return LORA_OK;
}

int32_t lora_slot_of(const lora_ctx* c, int32_t adapter_id)
{
    if (!c || adapter_id < 0 || adapter_id > c->cfg.max_adapter_id) return -1;
    return c->id2slot_h[adapter_id];
}

int32_t lora_slot_adapter(const lora_ctx* c, int32_t slot)
{
    if (!c || slot < 0 || slot >= c->cfg.n_slots) return -1;
    return c->slot_adapter[slot];
}

int32_t lora_slot_first_page(const lora_ctx* c, int32_t slot)
{
    if (!c || slot < 0 || slot >= c->cfg.n_slots || c->cfg.n_pages <= 0) return -1;
    return c->slot_first_page[slot];
}

lora_status lora_slots_load(lora_ctx* c, int32_t n, lora_adapter_desc* descs, const int32_t* in_use,
                            int32_t n_in_use, void* copy_stream_v)
{
    if (!c || n < 0 || n_in_use < 0 || (n > 0 && !descs) || (n_in_use > 0 && !in_use)) return LORA_ERR_INVALID_ARG;
    const int n_slots = c->cfg.n_slots, n_proj = c->cfg.n_proj;
    const int32_t max_id = c->cfg.max_adapter_id;

    // ---- validate ----
    for (int i = 0; i < n_in_use; ++i)
        if (in_use[i] < 0 || in_use[i] > max_id) return LORA_ERR_ID_RANGE;
    for (int i = 0; i < n; ++i) {
        const lora_adapter_desc& d = descs[i];
        if (d.adapter_id < 0 || d.adapter_id > max_id) return LORA_ERR_ID_RANGE;
        if (d.rank < 0) return LORA_ERR_INVALID_ARG;
        if (d.rank > c->cfg.max_rank) return LORA_ERR_RANK_EXCEEDS_SMAX;
        if (d.rank % 8) return LORA_ERR_SHAPE;
        if (d.slot < -1 || d.slot >= n_slots) return LORA_ERR_SLOT_RANGE;
        if (d.rank > 0 && !c->host_only) {
            if (!d.A || !d.B) return LORA_ERR_INVALID_ARG;
            for (int f = 0; f < n_proj * c->n_layers; ++f)
                if (!d.A[f] || !d.B[f]) return LORA_ERR_INVALID_ARG;
        }
    }

    // ---- plan on a copy of the table ----
    std::vector<int32_t> adapter = c->slot_adapter, rank = c->slot_rank_h, id2slot = c->id2slot_h;
    std::vector<float> scale = c->slot_scale_h;
    std::vector<uint64_t> last_used = c->slot_last_used;
    std::vector<int32_t> first_page = c->slot_first_page, owner = c->page_owner;
    const bool paged = c->cfg.n_pages > 0;
    const int n_pages = c->cfg.n_pages;
    const uint64_t tick = c->tick + 1;
    std::vector<char> is_protected((size_t)max_id + 1, 0), placed_now(n_slots, 0);
    for (int i = 0; i < n_in_use; ++i) {
        is_protected[in_use[i]] = 1;
        const int s = id2slot[in_use[i]];
        if (s >= 0) last_used[s] = tick;
    }
    struct Step { int slot, adapter, evicted, rank; float scale; bool copied; int first_page; };
    // paged slots: the pages of a slot go back to the pool; the lowest first page of a free run of k pages
    auto free_pages_of = [&](int slot) {
        if (!paged) return;
        first_page[slot] = -1;
        for (int p = 0; p < n_pages; ++p)
            if (owner[p] == slot) owner[p] = -1;
    };
    auto first_fit = [&](int k) {
        int run = 0;
        for (int p = 0; p < n_pages; ++p) {
            run = owner[p] < 0 ? run + 1 : 0;
            if (run == k) return p - k + 1;
        }
        return -1;
    };
    std::vector<Step> steps;
    steps.reserve(n);
    std::vector<int> out_slot(n), out_copied(n);
    for (int i = 0; i < n; ++i) {
        const lora_adapter_desc& d = descs[i];
        const int cur = id2slot[d.adapter_id];
        if (cur >= 0 && (d.slot < 0 || d.slot == cur)) {
            last_used[cur] = tick;
            placed_now[cur] = 1;
            out_slot[i] = cur;
            out_copied[i] = 0;
            continue;
        }
        int s = d.slot;
        if (s < 0) {
            for (int k = 0; k < n_slots && s < 0; ++k)
                if (adapter[k] < 0) s = k;
            if (s < 0) {
                uint64_t best = 0;
                for (int k = 0; k < n_slots; ++k) {
                    if (placed_now[k] || is_protected[adapter[k]]) continue;
                    if (s < 0 || last_used[k] < best) {
                        s = k;
                        best = last_used[k];
                    }
                }
                if (s < 0) return LORA_ERR_SLOTS_EXHAUSTED;
            }
        }
        if (cur >= 0) {  // the adapter moves to an explicit other slot: its old slot becomes empty
            steps.push_back({cur, -1, d.adapter_id, 0, 0.f, false, -1});
            adapter[cur] = -1;
            rank[cur] = 0;
            scale[cur] = 0.f;
            id2slot[d.adapter_id] = -1;
            free_pages_of(cur);
        }
        const int evicted = adapter[s];
        if (evicted >= 0) {
            id2slot[evicted] = -1;
            free_pages_of(s);
        }
        placed_now[s] = 1;
        int first = -1;
        if (paged && d.rank > 0) {
            // a run of rank / 8 pages, first fit; while there is none, further adapters leave in the order of slot
            // victims (not in use, not placed by this call, least recently used, lowest slot)
            const int need = d.rank / kPageRanks;
            first = first_fit(need);
            while (first < 0) {
                int v = -1;
                uint64_t best = 0;
                for (int k = 0; k < n_slots; ++k) {
                    if (adapter[k] < 0 || placed_now[k] || is_protected[adapter[k]]) continue;
                    if (v < 0 || last_used[k] < best) {
                        v = k;
                        best = last_used[k];
                    }
                }
                if (v < 0) return LORA_ERR_SLOTS_EXHAUSTED;
                steps.push_back({v, -1, adapter[v], 0, 0.f, false, -1});
                id2slot[adapter[v]] = -1;
                adapter[v] = -1;
                rank[v] = 0;
                scale[v] = 0.f;
                free_pages_of(v);
                first = first_fit(need);
            }
            for (int p = first; p < first + need; ++p) owner[p] = s;
            first_page[s] = first;
        }
        adapter[s] = d.adapter_id;
        rank[s] = d.rank;
        scale[s] = d.scale;
        id2slot[d.adapter_id] = s;
        last_used[s] = tick;
        placed_now[s] = 1;
        steps.push_back({s, d.adapter_id, evicted, d.rank, d.scale, true, first});
        out_slot[i] = s;
        out_copied[i] = 1;
    }

    // ---- commit ----
    c->slot_adapter.swap(adapter);
    c->slot_rank_h.swap(rank);
    c->slot_scale_h.swap(scale);
    c->slot_last_used.swap(last_used);
    c->id2slot_h.swap(id2slot);
    c->slot_first_page.swap(first_page);
    c->page_owner.swap(owner);
    c->tick = tick;
    c->n_resident = 0;
    for (int k = 0; k < n_slots; ++k) c->n_resident += c->slot_adapter[k] >= 0;
    for (int i = 0; i < n; ++i) {
        descs[i].slot = out_slot[i];
        descs[i].copied = out_copied[i];
    }
    if (c->host_only || steps.empty()) return LORA_OK;

    // ---- enqueue ----
    hipStream_t cs = static_cast<hipStream_t>(copy_stream_v);
    if (c->have_fwd && c->last_fwd_stream != cs) {
        // earlier steps may still read the slots about to be overwritten
        if (!c->fwd_marked && HIP_FAIL(hipEventRecord(c->ev_fwd, c->last_fwd_stream))) return LORA_ERR_HIP;
        if (HIP_FAIL(hipStreamWaitEvent(cs, c->ev_fwd, 0))) return LORA_ERR_HIP;
    }
    c->marks_left = kMarkedCallsPerLoad;
    for (size_t b = 0; b < steps.size(); b += kMetaBatch) {
        MetaUpdates u;
        std::memset(&u, 0, sizeof u);
        u.n = (int)std::min<size_t>(kMetaBatch, steps.size() - b);
        for (int i = 0; i < u.n; ++i) {
            const Step& st = steps[b + i];
            u.slot[i] = st.slot;
            u.adapter[i] = st.adapter;
            u.evicted[i] = st.evicted;
            u.rank[i] = st.rank;
            u.scale[i] = st.scale;
            u.loc[i] = st.adapter >= 0 ? c->loc_of(st.slot, st.first_page) : -1;
        }
        if (HIP_FAIL(launch_meta_update(u, c->d_slot_rank(), c->d_slot_scale(), c->d_slot_loc(), c->d_id2slot(), cs)))
            return LORA_ERR_HIP;
    }
    if (HIP_FAIL(hipEventRecord(c->ev_meta, cs))) return LORA_ERR_HIP;
    c->meta_pending = true;
    // The copies go out in units, in order: a unit is one projection, or one whole layer when the context holds
    // several layers (a forward pass running behind the copies can then start on the first layers while later
    // ones still travel); one event per unit.  Inside a slot an adapter's matrices follow each other without
    // gaps, so matrices that also follow each other in host memory travel as one run.
    // Two carriers.  A kernel that reads the pinned host memory itself, a batch of runs per launch: the faster
    // one on an idle GPU and for short runs (a copy call per run costs the host and the engine about 10 us), but
    // its workgroups find no free compute unit while forward kernels run.  The copy engine (hipMemcpyAsync per
    // run): needs no compute unit, so a load in the shadow of a running step keeps its rate.  Unless told
    // otherwise the engine carries a load whose runs all reach kEngineRunBytes (the matrices of a projection,
    // or whole layers, of an adapter kept as one host buffer), the kernel everything else; a source that is not
    // device-visible pinned host memory always goes through hipMemcpyAsync.
    char* slots = c->base + c->L.off_slots;
    const bool by_layer = c->n_layers > 1;
    const int n_units = by_layer ? c->n_layers : n_proj;
    struct Run { const char* src; char* dst; size_t bytes; };
    std::vector<std::vector<Run>> unit_runs(n_units);
    size_t shortest = SIZE_MAX;
    for (int u = 0; u < n_units; ++u) {
        const int f_begin = by_layer ? u * n_proj : u, f_end = by_layer ? (u + 1) * n_proj : u + 1;
        std::vector<Run>& runs = unit_runs[u];
        for (int i = 0; i < n; ++i) {
            if (!out_copied[i] || descs[i].rank <= 0) continue;
            // a later request of the same call may have taken the slot (an explicit slot overrides everything):
            // the adapter is then not resident and its place may belong to somebody else
            if (c->slot_adapter[out_slot[i]] != descs[i].adapter_id) continue;
            const size_t r = descs[i].rank;
            char* slot_base = slots + (size_t)c->loc_of(out_slot[i], c->slot_first_page[out_slot[i]]) * (kLocUnit * 2);
            const size_t first = runs.size();
            auto add = [&](const void* src, size_t dst_elems, size_t bytes) {
                const char* sp = static_cast<const char*>(src);
                char* dp = slot_base + dst_elems * 2;
                if (runs.size() > first) {
                    Run& last = runs.back();
                    if (sp == last.src + last.bytes && dp == last.dst + last.bytes && last.bytes + bytes <= 0xffffffffu) {
                        last.bytes += bytes;
                        return;
                    }
                }
                runs.push_back(Run{sp, dp, bytes});
            };
            for (int f = f_begin; f < f_end; ++f) {
                const int p = f % n_proj;
                add(descs[i].A[f], r * c->L.a_unit[f], r * (size_t)c->proj[p].d_in * 2);
                add(descs[i].B[f], r * c->L.b_unit[f], r * (size_t)c->proj[p].d_out * 2);
            }
        }
        for (const Run& r : runs) shortest = std::min(shortest, r.bytes);
    }
    const int tuned = c->tune[LORA_TUNE_COPY_ENGINE];
    const bool engine = tuned == LORA_COPY_ENGINE ||
                        (tuned != LORA_COPY_KERNEL && shortest >= kEngineRunBytes);
    for (int u = 0; u < n_units; ++u) {
        CopyBatch batch;
        batch.n = 0;
        auto flush = [&]() -> bool {
            if (batch.n > 0 && HIP_FAIL(launch_copy_batch(batch, cs))) return false;
            batch.n = 0;
            return true;
        };
        for (const Run& r : unit_runs[u]) {
            const void* dev_src = engine ? nullptr : device_view_of_pinned(r.src);
            const bool kernel_ok = dev_src && r.bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(r.src) & 15) == 0;
            if (!kernel_ok) {
                if (HIP_FAIL(hipMemcpyAsync(r.dst, r.src, r.bytes, hipMemcpyHostToDevice, cs))) return LORA_ERR_HIP;
                continue;
            }
            if (batch.n == kCopyBatch && !flush()) return LORA_ERR_HIP;
            batch.src[batch.n] = dev_src;
            batch.dst[batch.n] = r.dst;
            batch.bytes[batch.n] = (uint32_t)r.bytes;
            ++batch.n;
        }
        if (!flush()) return LORA_ERR_HIP;
        if (HIP_FAIL(hipEventRecord(c->ev_unit[u], cs))) return LORA_ERR_HIP;
        c->unit_pending[u] = 1;
    }
    c->copy_stream = cs;
    return LORA_OK;
}

lora_status lora_bucket(lora_ctx* c, const int32_t* d_token_adapter, int32_t T, int32_t mode, lora_segments* out,
                        void* stream_v)
{
    if (!c || !out || T < 0 || T > c->cfg.max_tokens) return LORA_ERR_INVALID_ARG;
    if (mode != LORA_BUCKET_SORTED && mode != LORA_BUCKET_RUNS) return LORA_ERR_INVALID_ARG;
    if (T > 0 && !d_token_adapter) return LORA_ERR_INVALID_ARG;
    if (c->host_only) return LORA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream_v);
    if (c->meta_pending && s != c->copy_stream) {
        if (HIP_FAIL(hipStreamWaitEvent(s, c->ev_meta, 0))) return LORA_ERR_HIP;
    }
    // the segment arrays are read by the forwards of the previous step: a map built on another stream waits for them
    if (c->have_fwd && c->last_fwd_stream != s) {
        if (HIP_FAIL(hipEventRecord(c->ev_fwd, c->last_fwd_stream))) return LORA_ERR_HIP;
        if (HIP_FAIL(hipStreamWaitEvent(s, c->ev_fwd, 0))) return LORA_ERR_HIP;
    }
    BucketArgs a;
    a.ids = d_token_adapter;
    a.T = T;
    a.mode = mode;
    a.id2slot = c->d_id2slot();
    a.n_ids = c->cfg.max_adapter_id + 1;
    a.n_slots = c->cfg.n_slots;
    a.perm = c->dev<int32_t>(c->L.off_perm);
    a.row_slot = c->dev<int32_t>(c->L.off_row_slot);
    a.row_rank = c->dev<int32_t>(c->L.off_row_rank);
    a.row_loc = c->dev<int32_t>(c->L.off_row_loc);
    a.slot_loc = c->d_slot_loc();
    a.row_scale = c->dev<float>(c->L.off_row_scale);
    a.slot_rank = c->d_slot_rank();
    a.slot_scale = c->d_slot_scale();
    a.seg_start = c->dev<int32_t>(c->L.off_seg_start);
    a.seg_slot = c->dev<int32_t>(c->L.off_seg_slot);
    a.n_seg = c->d_n_seg();
    a.piece_start = c->dev<int32_t>(c->L.off_piece_start);
    a.piece_slot = c->dev<int32_t>(c->L.off_piece_slot);
    a.n_pieces = c->d_n_pieces();
    a.piece_info = c->dev<int32_t>(c->L.off_piece_info);
    a.tok_key = c->dev<int32_t>(c->L.off_tok_key);
    a.flags = c->d_flags();
    c->last_launches.clear();
    {
        LaunchScope ls(c, s, "bucket");
        if (HIP_FAIL(launch_bucket(a, s))) return LORA_ERR_HIP;
    }
    c->epoch += 1;
    c->seg_T = T;
    c->seg_mode = mode;
    if (!c->work_enqueued(s)) return LORA_ERR_HIP;
    out->perm = a.perm;
    out->seg_start = a.seg_start;
    out->seg_slot = a.seg_slot;
    out->n_seg = a.n_seg;
    out->T = T;
    out->mode = mode;
    out->epoch = c->epoch;
    return LORA_OK;
}

}  // extern "C"

namespace {

// Where a forward call keeps its split-K partial tiles and shrink results: the context's slab, or the library's
// static array (lora_layer_forward_static).
struct ScratchRef {
    float* vpart;
    size_t vpart_elems;
    float* part;
    size_t part_elems;
    bool is_static;
};

// glu: the two projections are gate and up of the same tokens and silu(gate) * up is stored to d_out[0]
lora_status forward_impl(lora_ctx* c, int32_t layer, int32_t n, const int32_t* projs, const void* const* d_x,
                         const void* const* d_W, const lora_segments* seg, void* const* d_out, void* stream_v,
                         const ScratchRef& scr, bool glu = false)
{
    if (!c || !seg || !projs || n < 1 || n > kMaxGroup) return LORA_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->n_layers) return LORA_ERR_INVALID_ARG;
    const int flat0 = layer * c->cfg.n_proj;                 // this layer's projections in the per-layer tables
    for (int k = 0; k < n; ++k) {
        if (projs[k] < 0 || projs[k] >= c->cfg.n_proj) return LORA_ERR_INVALID_ARG;
        for (int j = 0; j < k; ++j)
            if (projs[j] == projs[k]) return LORA_ERR_INVALID_ARG;
        if (c->proj[projs[k]].d_in != c->proj[projs[0]].d_in) return LORA_ERR_SHAPE;
    }
    if (seg->epoch != c->epoch || seg->T != c->seg_T || c->epoch == 0) return LORA_ERR_INVALID_ARG;
    if (c->host_only) return LORA_ERR_HIP;
    const int32_t T = seg->T;
    c->last_launches.clear();
    if (T == 0) return LORA_OK;
    if (!d_x || !d_W || !d_out) return LORA_ERR_INVALID_ARG;
    for (int k = 0; k < n; ++k) {
        if (!d_x[k] || !d_W[k] || !d_out[k]) return LORA_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(d_x[k]) | reinterpret_cast<uintptr_t>(d_W[k]) |
             reinterpret_cast<uintptr_t>(d_out[k])) & 15)
            return LORA_ERR_INVALID_ARG;
    }
    hipStream_t s = static_cast<hipStream_t>(stream_v);
    // forwards (and segment maps) of one context share its scratch and its segment arrays: a call on another
    // stream than the previous one is ordered behind it
    if (c->have_fwd && c->last_fwd_stream != s) {
        if (HIP_FAIL(hipEventRecord(c->ev_fwd, c->last_fwd_stream))) return LORA_ERR_HIP;
        if (HIP_FAIL(hipStreamWaitEvent(s, c->ev_fwd, 0))) return LORA_ERR_HIP;
    }
    for (int k = 0; k < n; ++k) {
        const int u = c->unit_of(layer, projs[k]);
        if (c->unit_pending[u] && s != c->copy_stream && (k == 0 || u != c->unit_of(layer, projs[k - 1]))) {
            if (HIP_FAIL(hipStreamWaitEvent(s, c->ev_unit[u], 0))) return LORA_ERR_HIP;
        }
    }
    ForwardPlan plan;
    if (const lora_status st = plan_forward(c, T, n, projs, scr.part_elems, scr.vpart_elems, plan, glu); st != LORA_OK)
        return (st == LORA_ERR_OOM && scr.is_static) ? LORA_ERR_SCRATCH_LIMIT : st;
    const int K = plan.K, Mpad = plan.Mpad, S = plan.S, n_kc = plan.n_kc, kc_len = plan.kc_len;
    const long n_pad_total = plan.n_pad_total;
    const bool split = plan.split, dyn_shrink = plan.dyn_shrink;
    const int split_variant = plan.split_variant;
    auto tiles_of = [&](int bm, int bn) {
        long t = 0;
        for (int k = 0; k < n; ++k) t += (c->proj[projs[k]].d_out + bn - 1) / bn;
        return t * ((T + bm - 1) / bm);
    };
    const size_t vslice = (size_t)n_kc * T * c->cfg.max_rank;
    if (vslice * n > scr.vpart_elems) return scr.is_static ? LORA_ERR_SCRATCH_LIMIT : LORA_ERR_OOM;

    const DeviceView dv = c->view(T);
    float* vpart = scr.vpart;
    float* part = scr.part;

    GroupArgs g;
    std::memset(&g, 0, sizeof g);
    g.n = n;
    int blk = 0;
    for (int k = 0; k < n; ++k) {
        const int p = projs[k];
        Slice& sl = g.s[k];
        sl.x = static_cast<const uint16_t*>(d_x[k]);
        sl.W = static_cast<const uint16_t*>(d_W[k]);
        sl.out = static_cast<uint16_t*>(d_out[k]);
        sl.vpart = vpart + vslice * k;
        sl.a_unit = c->L.a_unit[flat0 + p];
        sl.b_unit = c->L.b_unit[flat0 + p];
        sl.bias = c->bias[flat0 + p];
        sl.N = c->proj[p].d_out;
        sl.tile0 = 0;
        sl.blk0 = blk;
        blk += (int)(align_up((size_t)sl.N, 128) / 32);
    }

    ShrinkArgs sa;
    std::memset(&sa, 0, sizeof sa);
    sa.dv = dv;
    sa.g = g;
    sa.K = K;
    sa.n_kc = n_kc;
    sa.kc_len = kc_len;
    sa.on = c->n_resident > 0 ? 1 : 0;      // no adapter resident: nothing to shrink

    GemmArgs ga;
    std::memset(&ga, 0, sizeof ga);
    ga.dv = dv;
    ga.g = g;
    ga.K = K;
    ga.split_k = S;
    ga.n_kc = n_kc;
    ga.nblk = blk;
    ga.part = part;
    ga.Mpad = Mpad;
    ga.m_begin = 0;
    ga.m_end = T;
    ga.main_grid = 0;
    ga.shrink_q = 0;
    if (split && dyn_shrink) {
        const int bm = split_bm(split_variant);
        const long main_wgs = tiles_of(bm, 128) * S;
        ga.main_grid = (int)std::max<long>(0, std::min<long>(c->n_cus / 2, c->n_cus - main_wgs));   // on entry: shrink-only workgroups
        // items a shrink-only workgroup finishes while a tile workgroup walks its K range: a 64-wide K tile of
        // the tile workgroup takes about 1 us, an item about 8
        const int nk = std::max(1, K / kBK / S);
        ga.shrink_q = std::max(1, nk / 4);
    }

    // split-K base GEMM (+ shrink items when shrink.on) over the rows of `a`, then reduce + expand
    auto launch_split = [&](const GemmArgs& a, const ShrinkArgs& shrink, int variant) -> lora_status {
        {
            LaunchScope ls(c, s, "gemm_splitk");
            const char* name = nullptr;
            // 6, 7: 64-wide K tiles; 8: the 32-wide 256 x 128 kernel (its own variant 0); 1 .. 5: 32-wide variants
            const hipError_t le = (variant == 6 || variant == 7 || variant == 9)
                                      ? launch_gemm_rows128_splitk(a, shrink, variant == 9 ? 2 : variant - 6, s, &name)
                                      : launch_gemm_splitk(a, shrink, variant == 8 ? 0 : variant, s, &name);
            if (HIP_FAIL(le)) return LORA_ERR_HIP;
            ls.rename(name);
        }
        ReduceArgs ra;
        std::memset(&ra, 0, sizeof ra);
        ra.dv = dv;
        ra.g = g;
        ra.split_k = a.split_k;
        ra.Mpad = a.Mpad;
        ra.nblk = blk;
        ra.part = part;
        ra.n_kc = n_kc;
        ra.m_begin = a.m_begin;
        ra.m_end = a.m_end;
        const int grid = ((a.m_end - a.m_begin + kPieceRows - 1) / kPieceRows) * (blk / 4);
        LaunchScope ls(c, s, "reduce_expand");
        if (HIP_FAIL(launch_reduce_expand(ra, grid, s))) return LORA_ERR_HIP;
        return LORA_OK;
    };

    if (!split) {
        // ---- shrink, then base GEMM with the expand in its epilogue ----
        int fv = c->tune[LORA_TUNE_FUSED_VARIANT];
        const bool auto_variant = fv == 0 && !glu;
        // gate and up with their product: the 64-wide-K kernel up to 1024 tokens (128-row tiles up to 128), the
        // register-staged 256 x 256 tile above
        if (glu) fv = T <= 128 ? 9 : (T <= kSplitMaxTokens ? 8 : 0);
        if (auto_variant) {
            fv = pick_fused_variant(c->n_cus, tiles_of);
            // small batch: bound by the copies, not by the MFMA issue: whole-line tiles, every wave copies
            // (128-row tiles up to 128 tokens)
            if (T <= kSplitMaxTokens) fv = T <= 128 ? 9 : (fv == 4 ? 8 : (fv == 3 ? 9 : 10));
            // between 129 and 1024 tokens the launch is bound by what a workgroup moves through its CU: rounds
            // of workgroups over the CUs times the rows (x and W) of a tile; near ties go to the larger tile
            if (T > 128 && T <= kSplitMaxTokens) {
                const struct { int v, bm, bn; } cand[] = {{10, 256, 256}, {11, 256, 192}, {8, 256, 128}, {9, 128, 128}};
                double best = 0.0;
                for (const auto& cd : cand) {
                    const double cost = (double)((tiles_of(cd.bm, cd.bn) + c->n_cus - 1) / c->n_cus) * (cd.bm + cd.bn);
                    if (best == 0.0 || cost < best * 0.97) {
                        best = cost;
                        fv = cd.v;
                    }
                }
            }
        }
        // A last round of 256 x 256 tiles that fills less than half the chip costs as much as a full one.  When
        // the rows behind the full rounds are few enough for the split-K path, the fused launch stops at the
        // full rounds and those rows take the split-K path (their shrink results are there already), which
        // spreads them over every CU.
        int m_split = T;
        int tail_S = 1;
        if (auto_variant && fv == 0 && c->cfg.path == LORA_PATH_AUTO && T > kSplitMaxTokens) {
            const long tiles_m_big = (T + 255) / 256, tiles_big = tiles_of(256, 256), tiles_n_big = tiles_big / tiles_m_big;
            const long full = tiles_big / c->n_cus, rest = tiles_big % c->n_cus;
            if (full >= 1 && rest > 0 && rest <= c->n_cus / 2) {
                const long m_tiles_main = std::min(tiles_m_big - 1, full * c->n_cus / tiles_n_big);
                const long tail_rows = (long)T - m_tiles_main * 256;
                if (m_tiles_main >= 1 && tail_rows > 0 && tail_rows <= kSplitMaxTokens) {
                    long tail_tiles = 0;
                    for (int k = 0; k < n; ++k) tail_tiles += (c->proj[projs[k]].d_out + 127) / 128;
                    tail_tiles *= (tail_rows + 255) / 256;
                    const long tail_pad = (tail_rows + 255) / 256 * 256;
                    long ts = std::max<long>(1, std::min<long>(8, (c->n_cus + tail_tiles / 2) / tail_tiles));
                    ts = std::min<long>(ts, std::max(1, (K / kBK) / 2));
                    ts = std::min<long>(ts, (long)(scr.part_elems / ((size_t)tail_pad * (size_t)n_pad_total)));
                    if (ts >= 2) {
                        m_split = (int)(m_tiles_main * 256);
                        tail_S = (int)ts;
                    }
                }
            }
        }
        // Small batches leave CUs without a tile (224 tiles of 256 x 128 for a Llama-8B gate|up, 198 of 256 x 192
        // for Qwen2.5-7B).  When those CUs can finish the shrink well inside the time the tiles stream, they do
        // it as the first workgroups of the GEMM launch and the separate shrink launch goes.
        int front = 0;
        if (sa.on && fv >= 8 && fv <= 11 && T <= kSplitMaxTokens && m_split == T && !c->inline_shrink_off &&
            c->tune[LORA_TUNE_INLINE_SHRINK] != LORA_INLINE_SHRINK_OFF) {
            const int bm = fv == 9 ? 128 : 256, bn = fv == 10 ? 256 : (fv == 11 ? 192 : 128);
            const long idle = c->n_cus - tiles_of(bm, bn);
            // unsplit up to K = 4096 (two rounds of loads per item): the tile workgroups then fetch one partial
            // result per row instead of two, behind their last K tile
            const int chunks = std::max(1, std::min<int>(kMaxShrinkChunks, K / 4096));
            const long pieces = (long)n * std::min<long>(T, (long)c->n_resident + (T + kPieceRows - 1) / kPieceRows);
            const double t_main = (double)(bm + bn) * K * 2.0 / 48e3;                   // us, see plan_forward
            if (idle >= 8 && chunks <= n_kc &&      // the scratch for the shrink results is sized for n_kc chunks
                (c->tune[LORA_TUNE_INLINE_SHRINK] == LORA_INLINE_SHRINK_ON ||
                 (double)(pieces * chunks) * (4.0 * (K / chunks) / 2048.0) / (double)std::min<long>(idle, c->n_cus / 4) <= 0.6 * t_main)) {
                front = (int)std::min<long>(idle, c->n_cus / 4);
                sa.n_kc = chunks;
                sa.kc_len = ((K + chunks - 1) / chunks + kBK - 1) / kBK * kBK;
                sa.n_kc = (K + sa.kc_len - 1) / sa.kc_len;
                ga.n_kc = sa.n_kc;
            }
        }
        if (sa.on && front == 0) {
            const long seg_bound = seg->mode == LORA_BUCKET_SORTED ? std::min<long>(T, (long)c->cfg.n_slots + 1) : T;
            const long items = (seg_bound + (T + kPieceRows - 1) / kPieceRows) * n_kc * n;
            const int grid = (int)std::max<long>(1, std::min<long>(items, 4096));
            LaunchScope ls(c, s, "shrink");
            if (HIP_FAIL(launch_shrink(sa, grid, s))) return LORA_ERR_HIP;
        }
        {
            LaunchScope ls(c, s, "gemm_fused");
            const char* name = nullptr;
            GemmArgs a = ga;
            a.m_end = m_split;
            a.shrink_front = front;
            // LORA_TUNE_SHRINK_WAIT_TEST: the tile workgroups expect one report more than will come and give up
            // after that many polls (host-forced exercise of the expired wait; every kernel still ends normally)
            const int wait_test = c->tune[LORA_TUNE_SHRINK_WAIT_TEST];
            a.front_expect = front + (wait_test > 0 && front > 0 ? 1 : 0);
            a.wait_spins = wait_test > 0 ? wait_test : kShrinkWaitSpins;
            a.sync = c->dev<uint32_t>(c->L.off_header) + 8;
            a.flags = c->d_flags();
            // 8 .. 11, 13, 14: 64-wide K tiles through the copy instruction; 12: the 32-wide 256 x 256 eight-wave kernel
            const hipError_t le = glu ? (fv == 0 ? launch_gemm_staged_glu(a, s, &name) : launch_gemm_rows128_glu(a, sa, fv - 8, s, &name))
                                  : ((fv >= 8 && fv <= 11) || fv == 13 || fv == 14)
                                      ? launch_gemm_rows128_fused(a, sa, fv >= 13 ? fv - 9 : fv - 8, s, &name)
                                      // 0 (the big tile of the automatic choice), 15, 16: tiles staged through registers
                                      : (fv == 0 || (fv >= 15 && fv <= 18)) ? launch_gemm_staged_fused(a, fv == 0 ? 0 : fv - 15, s, &name)
                                                                          : launch_gemm_fused(a, fv == 12 ? 0 : fv, s, &name);
            if (HIP_FAIL(le)) return LORA_ERR_HIP;
            ls.rename(name);
        }
        if (m_split < T) {
            GemmArgs a = ga;
            a.m_begin = m_split;
            a.m_end = T;
            a.split_k = tail_S;
            a.Mpad = (T - m_split + 255) / 256 * 256;
            ShrinkArgs none = sa;
            none.on = 0;
            const lora_status st = launch_split(a, none, 6);
            if (st != LORA_OK) return st;
        }
    } else {
        const lora_status st = launch_split(ga, sa, split_variant);
        if (st != LORA_OK) return st;
    }
    if (!c->work_enqueued(s)) return LORA_ERR_HIP;
    return LORA_OK;
}

ScratchRef slab_scratch(const lora_ctx* c)
{
    if (!c || c->host_only) return ScratchRef{nullptr, 0, nullptr, 0, false};
    return ScratchRef{c->dev<float>(c->L.off_vpart), c->L.vpart_elems, c->dev<float>(c->L.off_part), c->L.part_elems, false};
}

}  // namespace

extern "C" {

lora_status lora_model_forward_group(lora_ctx* c, int32_t layer, int32_t n, const int32_t* projs,
                                     const void* const* d_x, const void* const* d_W, const lora_segments* seg,
                                     void* const* d_out, void* stream_v)
{
    return forward_impl(c, layer, n, projs, d_x, d_W, seg, d_out, stream_v, slab_scratch(c));
}

lora_status lora_layer_forward_static(lora_ctx* c, int32_t p, const void* d_x, const void* d_W, const lora_segments* seg,
                                      void* d_out, void* stream_v)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    if (c->host_only || !c->static_scratch) return LORA_ERR_HIP;
    ScratchRef scr;
    scr.part = reinterpret_cast<float*>(c->static_scratch);
    scr.part_elems = kStaticPartBytes / 4;
    scr.vpart = reinterpret_cast<float*>(c->static_scratch + kStaticPartBytes);
    scr.vpart_elems = kStaticVpartBytes / 4;
    scr.is_static = true;
    return forward_impl(c, 0, 1, &p, &d_x, &d_W, seg, &d_out, stream_v, scr);
}

size_t lora_static_scratch_bytes(void) { return kStaticPartBytes + kStaticVpartBytes; }

lora_status lora_model_forward_glu(lora_ctx* c, int32_t layer, int32_t proj_gate, int32_t proj_up, const void* d_x,
                                   const void* d_W_gate, const void* d_W_up, const lora_segments* seg, void* d_out,
                                   void* stream_v)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->n_layers) return LORA_ERR_INVALID_ARG;
    if (proj_gate < 0 || proj_gate >= c->cfg.n_proj || proj_up < 0 || proj_up >= c->cfg.n_proj || proj_gate == proj_up)
        return LORA_ERR_INVALID_ARG;
    if (c->proj[proj_gate].d_out != c->proj[proj_up].d_out || c->proj[proj_gate].d_in != c->proj[proj_up].d_in)
        return LORA_ERR_SHAPE;
    const size_t flat0 = (size_t)layer * c->cfg.n_proj;
    if (c->bias[flat0 + proj_gate] || c->bias[flat0 + proj_up]) return LORA_ERR_INVALID_ARG;      // the gated MLPs served here have none
    const int32_t projs[2] = {proj_gate, proj_up};
    const void* xs[2] = {d_x, d_x};
    const void* Ws[2] = {d_W_gate, d_W_up};
    void* outs[2] = {d_out, d_out};
    return forward_impl(c, layer, 2, projs, xs, Ws, seg, outs, stream_v, slab_scratch(c), true);
}

lora_status lora_layer_forward_glu(lora_ctx* c, int32_t proj_gate, int32_t proj_up, const void* d_x, const void* d_W_gate,
                                   const void* d_W_up, const lora_segments* seg, void* d_out, void* stream_v)
{
    return lora_model_forward_glu(c, 0, proj_gate, proj_up, d_x, d_W_gate, d_W_up, seg, d_out, stream_v);
}

lora_status lora_layer_forward_group(lora_ctx* c, int32_t n, const int32_t* projs, const void* const* d_x,
                                     const void* const* d_W, const lora_segments* seg, void* const* d_out,
                                     void* stream_v)
{
    return lora_model_forward_group(c, 0, n, projs, d_x, d_W, seg, d_out, stream_v);
}

lora_status lora_layer_forward(lora_ctx* c, int32_t p, const void* d_x, const void* d_W, const lora_segments* seg,
                               void* d_out, void* stream_v)
{
    return lora_model_forward_group(c, 0, 1, &p, &d_x, &d_W, seg, &d_out, stream_v);
}

lora_status lora_poll_device_flags(lora_ctx* c, uint32_t* flags, void* stream_v)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    if (c->host_only) return LORA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream_v);
    uint32_t word = 0;
    if (HIP_FAIL(hipMemcpyAsync(&word, c->d_flags(), sizeof word, hipMemcpyDeviceToHost, s))) return LORA_ERR_HIP;
    if (HIP_FAIL(launch_fill_i32(reinterpret_cast<int32_t*>(c->d_flags()), 0, 1, s))) return LORA_ERR_HIP;
    if (HIP_FAIL(hipStreamSynchronize(s))) return LORA_ERR_HIP;
    if (flags) *flags = word;
    if (word & LORA_FLAG_INTERNAL) {
        // a bounded wait inside a kernel expired: the counters it used may be left half-way, and the assumption
        // the wait rests on (the launch's first workgroups run first) failed once: no more shrink inside a launch
        c->inline_shrink_off = true;
        if (HIP_FAIL(launch_fill_i32(c->dev<int32_t>(c->L.off_header) + 8, 0, 2, s))) return LORA_ERR_HIP;
        if (HIP_FAIL(hipStreamSynchronize(s))) return LORA_ERR_HIP;
        g_last_hip_error = "a kernel's bounded wait for the launch's shrink workgroups expired";
        return LORA_ERR_HIP;
    }
    return (word & LORA_FLAG_NOT_RESIDENT) ? LORA_ERR_NOT_RESIDENT : LORA_OK;
}

lora_status lora_set_bias(lora_ctx* c, int32_t layer, int32_t proj, const void* d_bias)
{
    if (!c || proj < 0 || proj >= c->cfg.n_proj || layer < 0 || layer >= c->n_layers) return LORA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_bias) & 15) return LORA_ERR_INVALID_ARG;
    c->bias[(size_t)layer * c->cfg.n_proj + proj] = static_cast<const uint16_t*>(d_bias);
    return LORA_OK;
}

lora_status lora_set_tuning(lora_ctx* c, int32_t key, int32_t value)
{
    if (!c || key < 0 || key >= 8) return LORA_ERR_INVALID_ARG;
    c->tune[key] = value;
    return LORA_OK;
}

int32_t lora_last_launches(const lora_ctx* c, const char** names, int32_t cap)
{
    if (!c) return 0;
    const int32_t n = (int32_t)c->last_launches.size();
    for (int32_t i = 0; i < n && i < cap && names; ++i) names[i] = c->last_launches[i];
    return n;
}

lora_status lora_profile_enable(lora_ctx* c, int32_t on)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    if (c->host_only) return LORA_ERR_HIP;
    if (on && c->prof_pool.empty()) {
        c->prof_pool.resize(8192);
        for (auto& sl : c->prof_pool) {
            sl.name = nullptr;
            if (HIP_FAIL(hipEventCreate(&sl.beg)) || HIP_FAIL(hipEventCreate(&sl.end))) return LORA_ERR_HIP;
        }
    }
    c->profiling = on != 0;
    return LORA_OK;
}

int32_t lora_profile_collect(lora_ctx* c, const char** names, double* total_ms, int64_t* counts, int32_t cap)
{
    if (!c || c->host_only) return 0;
    for (size_t i = 0; i < c->prof_used; ++i) {
        ProfileSlot& sl = c->prof_pool[i];
        float ms = 0.f;
        if (HIP_FAIL(hipEventSynchronize(sl.end))) continue;
        if (HIP_FAIL(hipEventElapsedTime(&ms, sl.beg, sl.end))) continue;
        size_t k = 0;
        for (; k < c->prof_names.size(); ++k)
            if (c->prof_names[k] == sl.name) break;
        if (k == c->prof_names.size()) {
            c->prof_names.emplace_back(sl.name);
            c->prof_ms.push_back(0.0);
            c->prof_count.push_back(0);
        }
        c->prof_ms[k] += ms;
        c->prof_count[k] += 1;
    }
    c->prof_used = 0;
    const int32_t n = (int32_t)c->prof_names.size();
    for (int32_t k = 0; k < n && k < cap; ++k) {
        if (names) names[k] = c->prof_names[k].c_str();
        if (total_ms) total_ms[k] = c->prof_ms[k];
        if (counts) counts[k] = c->prof_count[k];
    }
    return n;
}

lora_status lora_profile_reset(lora_ctx* c)
{
    if (!c) return LORA_ERR_INVALID_ARG;
    c->prof_used = 0;
    c->prof_names.clear();
    c->prof_ms.clear();
    c->prof_count.clear();
    return LORA_OK;
}

}  // extern "C"
