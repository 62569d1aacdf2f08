/*
 * liblora_mi355 - one serving step of a shared LLM backbone with many unmerged LoRA
 * adapters, for AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * Problem statement followed (paper Sec. 1 and Sec. 2.2): adapters are kept unmerged over one
 * shared backbone; a LoRA adapter is two low-rank matrices per targeted layer whose activations
 * are added to the backbone layer's output, its size being its rank; requests of different
 * adapters run inside the same batch; a request can run only while its adapter is in GPU memory;
 * the GPU holds a fixed region of at most A_max adapters, each slot sized for the largest
 * adapter (S_max), and adapters are swapped in from CPU memory.  Sec. 2.1: one step mixes
 * prefill tokens with one-token decode requests (continuous batching).
 *
 * Per token t with adapter i = id[t], every targeted projection p computes
 *
 *     y[t,:] = x[t,:] W_p^T + s_i (x[t,:] A_{i,p}^T) B_{i,p}^T        (id[t] = -1: backbone only)
 *
 * with W_p [d_out,d_in], A_{i,p} [r_i,d_in], B_{i,p} [d_out,r_i], all row-major bf16, s_i fp32;
 * products are accumulated in fp32 and y is rounded once to bf16 (nearest even).
 *
 * Conventions for every call
 *   - returns a lora_status, never throws, never aborts the process;
 *   - "device" pointers are HIP device memory of the current device, "host" pointers are
 *     ordinary process memory, "pinned host" is page-locked memory from hipHostMalloc;
 *   - argument errors are detected on the host and reported before anything is enqueued;
 *   - GPU work is enqueued on the stream handed in (a hipStream_t passed as void*; NULL = the
 *     default stream); no hot call (lora_slots_load, lora_bucket, lora_layer_forward)
 *     synchronises with the device or allocates device memory (lora_slots_load plans on small
 *     host-side copies of the slot table and asks the runtime about each pinned source buffer);
 *   - there is no CPU fallback: without a usable GPU the calls that enqueue work fail with
 *     LORA_ERR_HIP.
 */
#ifndef LORA_MI355_H
#define LORA_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lora_ctx lora_ctx; /* opaque */

typedef enum {
    LORA_OK = 0,
    LORA_ERR_INVALID_ARG = 1,      /* null pointer, negative size, unknown mode, stale segment map */
    LORA_ERR_SHAPE = 2,            /* unsupported projection shape or rank (see lora_create) */
    LORA_ERR_OOM = 3,              /* the memory handed in is smaller than lora_slab_bytes() */
    LORA_ERR_SLOT_RANGE = 4,       /* explicit slot index outside [0, n_slots) */
    LORA_ERR_RANK_EXCEEDS_SMAX = 5,/* adapter rank larger than max_rank (S_max) */
    LORA_ERR_SLOTS_EXHAUSTED = 6,  /* every slot is held by an adapter of the current batch */
    LORA_ERR_NOT_RESIDENT = 7,     /* reported by lora_poll_device_flags: a token named a non-resident adapter */
    LORA_ERR_HIP = 8,              /* a HIP runtime call failed (no device, bad stream, ...) */
    LORA_ERR_ID_RANGE = 9,         /* adapter id outside [0, max_adapter_id] */
    LORA_ERR_STARVATION = 10,      /* lora_place_adapters: no starvation-free allocation on the GPUs given */
    LORA_ERR_SCRATCH_LIMIT = 11    /* lora_layer_forward_static: the call needs more scratch than the static buffer holds */
} lora_status;

/* Segment-map modes (lora_bucket). */
enum {
    LORA_BUCKET_SORTED = 0, /* group tokens by slot with a stable sort: decode / mixed steps */
    LORA_BUCKET_RUNS = 1    /* keep token order, segments = runs of equal slot: prefill, tokens contiguous per request */
};

/* Kernel-path override for lora_layer_forward (lora_config.path). */
enum {
    LORA_PATH_AUTO = 0,  /* chosen from T and the projection shape */
    LORA_PATH_FUSED = 1, /* one GEMM pass over full K, LoRA expand inside its epilogue */
    LORA_PATH_SPLITK = 2 /* K split over workgroups, fp32 partials, reduce + expand kernel */
};

/* Bits of the device flag word (lora_poll_device_flags). */
enum {
    LORA_FLAG_NOT_RESIDENT = 1u,
    LORA_FLAG_INTERNAL = 2u /* a bounded wait inside a kernel expired (never seen; a safety net): the results of
                               the calls since the last poll are invalid, lora_poll_device_flags returns LORA_ERR_HIP */
};

/* lora_config.flags */
enum {
    LORA_CREATE_HOST_ONLY = 1u /* slot-table bookkeeping only: no device memory, nothing enqueued
                                  (lets a scheduler or simulator replay the adapter cache) */
};

typedef struct {
    int32_t d_in;  /* multiple of 64 */
    int32_t d_out; /* multiple of 8 */
} lora_proj_shape;

typedef struct {
    int32_t n_slots;        /* A_max: adapters resident at once, 1 .. 4095 */
    int32_t max_rank;       /* S_max: slot size in rank units, multiple of 8, 8 .. 64 */
    int32_t n_proj;         /* targeted projections per layer, 1 .. 16 */
    const lora_proj_shape *proj; /* host, n_proj entries, copied by lora_create */
    int32_t max_tokens;     /* largest T of any step; max_tokens * d_in and d_out * d_in must stay below 2^32 */
    int32_t max_adapter_id; /* adapter ids are 0 .. max_adapter_id */
    void *slab;             /* device memory owned by the caller, 256-byte aligned, lora_slab_bytes() long;
                               holds the slot region and all scratch; must outlive the context */
    size_t slab_bytes;
    int32_t path;           /* LORA_PATH_* */
    int32_t split_k;        /* 0 = automatic; otherwise the K split of the SPLITK path (1..16) */
    uint32_t flags;         /* LORA_CREATE_* */
    int32_t n_layers;       /* decoder layers that share the slot table, 1 .. 256 (0 is read as 1): a slot then
                               holds one adapter's matrices for every layer, see lora_model_forward_group */
    int32_t n_pages;        /* 0: every slot owns room for an adapter of max_rank (the uniform footprint of the paper's
                               setting, Sec. 2.2 / 8.1).  > 0: the adapters share a pool of n_pages pages of 8 rank
                               units each (unified paging, Sec. 2.2): an adapter of rank r takes r / 8 consecutive
                               pages wherever a run is free, and a slot is an entry of a table that says where.
                               At least max_rank / 8; the slab is sized for the pool instead of n_slots regions. */
} lora_config;

/* One adapter to make resident.  A[p] / B[p]: pinned host, row-major bf16, A[p] is
 * [rank, d_in_p], B[p] is [d_out_p, rank]; they must stay valid and unchanged until the copy
 * stream has passed the call.  With n_layers > 1 the arrays hold n_layers * n_proj pointers,
 * layer-major: A[layer * n_proj + p].  Inside its slot an adapter is stored packed at its own
 * rank in the order A[0], B[0], A[1], B[1], ...: matrices that follow each other in that order
 * in host memory too (an adapter kept as one buffer) travel as one copy per projection, or per
 * layer when n_layers > 1.  rank must be 0 or a multiple of 8 (<= max_rank); rank 0 needs no
 * A/B.  slot: in, >= 0 = explicit slot, -1 = the library picks (an empty slot, else the least
 * recently used one); out = slot used.  copied: out, 1 if weights were copied, 0 if the adapter
 * was already resident (touch only). */
typedef struct {
    int32_t adapter_id;
    int32_t rank;
    float scale;            /* s_i = alpha / rank */
    int32_t slot;
    int32_t copied;
    const void *const *A;
    const void *const *B;
} lora_adapter_desc;

/* Result of lora_bucket.  The arrays are device memory owned by the context and stay valid
 * until the next lora_bucket on it.  perm[T]: token index at each grouped position;
 * seg_start[n_seg+1], seg_slot[n_seg]: segment g covers grouped positions
 * [seg_start[g], seg_start[g+1]) and uses slot seg_slot[g] (-1 = backbone only);
 * n_seg: one int32.  Entries past n_seg are unspecified. */
typedef struct {
    const int32_t *perm;
    const int32_t *seg_start;
    const int32_t *seg_slot;
    const int32_t *n_seg;
    int32_t T;
    int32_t mode;
    uint64_t epoch; /* identifies the lora_bucket call that produced this map */
} lora_segments;

/* Device bytes the context needs for `cfg` (slot region + scratch); 0 if cfg is invalid.  Paper Sec. 2.2: the
 * serving engine reserves a fixed GPU region for at most A_max simultaneously loaded adapters, each slot sized for
 * the largest adapter (S_max; Sec. 8.1 sets S_max to the largest adapter of the scenario).
 * Slot region = n_slots * n_layers * max_rank * sum_p (d_in_p + d_out_p) * 2 bytes: every slot has the
 * uniform S_max footprint, but kernels only ever read an adapter's own rank rows.  The scratch behind it is
 * sized for the compute units of the current device: query on the device the context will be created on. */
size_t lora_slab_bytes(const lora_config *cfg);

/* Creates a context on the current device: the adapter cache of one serving instance (paper Sec. 2.2: A_max slots
 * of S_max, adapters swapped in from CPU memory; Sec. 8.1: one instance per GPU) together with the scratch of its
 * projection calls.  cfg->slab must hold lora_slab_bytes(cfg) bytes (LORA_ERR_OOM otherwise).  All slots start
 * empty.  One context serves one stream of steps: calls on it are not thread-safe, and its forward calls and
 * segment maps share scratch (see lora_layer_forward).  Errors: INVALID_ARG, SHAPE, OOM, HIP. */
lora_status lora_create(const lora_config *cfg, lora_ctx **out);

/* Ends the adapter cache (paper Sec. 2.2; unloading costs nothing, Sec. 5.2): waits for the device, releases the
 * context's events and host tables.  The slab stays the caller's.  Errors: INVALID_ARG (NULL). */
lora_status lora_destroy(lora_ctx *ctx);

/* Makes n adapters resident (paper Sec. 2.2 / Sec. 5.1.3: adapters are loaded from CPU memory
 * into the GPU's adapter region; load time grows with adapter size, unloading is free).
 * in_use / n_in_use (host): adapter ids of the batch about to run; they are marked used now and
 * are never chosen as victims.  The whole call is planned on the host first: on any error
 * nothing is enqueued and the table is unchanged.  On success the slot metadata update, the
 * id->slot map update and the copies are enqueued on copy_stream, the copies projection after
 * projection (layer after layer when n_layers > 1) with one event each.  Runs travel in launches
 * of a kernel that reads the page-locked host buffers directly, or, when every run of the call
 * is at least 128 KiB, through the copy engine, which keeps its rate while forward
 * kernels occupy the compute units (LORA_TUNE_COPY_ENGINE overrides the choice; a source that is not
 * page-locked, device-visible host memory is always copied with hipMemcpyAsync).  Later
 * lora_bucket / lora_layer_forward calls on other streams wait through those events, each
 * forward only for the copies of its own projection (layer), and the copies themselves wait
 * for forward work of this context already enqueued (a slot is never overwritten while an earlier step may
 * still read it: forward calls of a context are chained across streams, see lora_layer_forward, so the wait for
 * the latest one covers all of them; work that other contexts have enqueued on the same stream since is not
 * waited for once the context has loaded before).  With n_pages > 0 a load may also send away adapters that the
 * call does not name, to free a run of pages (see lora_config.n_pages).
 * Errors: INVALID_ARG, ID_RANGE, SLOT_RANGE, RANK_EXCEEDS_SMAX, SHAPE (rank not a multiple of
 * 8), SLOTS_EXHAUSTED, HIP. */
lora_status lora_slots_load(lora_ctx *ctx, int32_t n, lora_adapter_desc *descs,
                            const int32_t *in_use, int32_t n_in_use, void *copy_stream);

/* Builds the token->adapter segment map for one step (shared by all projections and layers
 * of the step).  Paper Sec. 2.2: requests of different adapters run inside the same batch (each adapter's
 * matrices are then streamed once per step, for the tokens that use it); Sec. 2.1: a step mixes the tokens of
 * prefill chunks with one-token decode requests; Sec. 2.2: a request can run only while its adapter is in GPU
 * memory (hence the residency flag).  d_token_adapter: device, int32[T], adapter id per token or -1.  Integer work
 * only; the result is unique: SORTED = stable ascending sort of token indices by slot (slot -1
 * first) + run-length encoding; RUNS = identity order + run-length encoding.  A token whose
 * adapter id is out of range or not resident sets LORA_FLAG_NOT_RESIDENT in the device flag
 * word and is treated as -1.  T = 0 is valid (n_seg = 0).  The map replaces the previous one: when `stream` is
 * not the stream of the context's previous forward call, the library first orders it behind that call.
 * Errors: INVALID_ARG (T < 0, T > max_tokens, bad mode, null pointers), HIP. */
lora_status lora_bucket(lora_ctx *ctx, const int32_t *d_token_adapter, int32_t T, int32_t mode,
                        lora_segments *out, void *stream);

/* One projection of the step: d_out[t,:] = bf16(x[t,:] W^T + s (x[t,:] A^T) B^T) for every token,
 * in original token order (paper Sec. 2.2: a LoRA adapter is two low-rank matrices per targeted layer whose
 * activations are added to the backbone layer's output; Sec. 1: adapters stay unmerged over one shared backbone).
 * d_x: device bf16 [T, d_in_p]; d_W: device bf16 [d_out_p, d_in_p];
 * d_out: device bf16 [T, d_out_p]; all row-major, 16-byte aligned, not aliased.  seg must be
 * the map of the latest lora_bucket on this context.  T = 0 is a no-op.
 * Stream ordering: all forward calls (and segment maps) of one context share its scratch (split-K partial tiles,
 * shrink results, the counters of a launch), so they must not overlap in time.  The library sees to that itself:
 * a call whose stream differs from the stream of the context's previous lora_bucket / forward call is ordered
 * behind it with an event before anything is enqueued.  Calls that should run concurrently need contexts of
 * their own.  When the call uses the shrink inside its launch and lora_poll_device_flags later reports
 * LORA_FLAG_INTERNAL, the outputs written since the previous poll are undefined.
 * Errors: INVALID_ARG (proj out of range, stale seg, null or misaligned pointers), HIP. */
lora_status lora_layer_forward(lora_ctx *ctx, int32_t proj, const void *d_x, const void *d_W,
                               const lora_segments *seg, void *d_out, void *stream);

/* lora_layer_forward for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and
 * same kernels as lora_layer_forward, but the scratch of the call (split-K partial tiles, shrink results) lives in
 * a buffer of lora_static_scratch_bytes() = 40 MiB that is part of the library image, one copy per GPU, held
 * until the process ends, instead of the context's slab.  The call allocates nothing and frees nothing.  A call
 * whose shrink results do not fit (more than 2 Mi values: tokens x max_rank x K chunks) or whose partial tiles do
 * not fit even unsplit (more than 8 Mi values: tokens rounded up to 256 x d_out rounded up to 128) fails with
 * LORA_ERR_SCRATCH_LIMIT before anything is enqueued; between those limits the K split shrinks to what fits, so
 * the rounding order, not the tolerance, may differ from lora_layer_forward.  Nothing in the buffer has to start
 * at zero: every value a call reads it has written itself.  All calls on one GPU, from every context, share the
 * one buffer: two such calls that overlap in time on a GPU race; order them on one stream or by events.
 * Errors: as lora_layer_forward, plus SCRATCH_LIMIT. */
lora_status lora_layer_forward_static(lora_ctx *ctx, int32_t proj, const void *d_x, const void *d_W,
                                      const lora_segments *seg, void *d_out, void *stream);
size_t lora_static_scratch_bytes(void);

/* Packed projections (paper Sec. 2.2 applied to projections that are computed from one layer input side by
 * side, such as q|k|v and gate|up): the same result as n calls of lora_layer_forward for projs[0..n-1] in
 * order, served by shared launches.  1 <= n <= 4, the projections must be distinct and share d_in
 * (LORA_ERR_SHAPE otherwise); d_x[k], d_W[k], d_out[k] are the device pointers of projection projs[k] (the x
 * pointers may be equal or different), layouts and alignment as for lora_layer_forward; the three pointer
 * arrays live in host memory and are read before the call returns.  Asynchronous on `stream`. */
lora_status lora_layer_forward_group(lora_ctx* ctx, int32_t n, const int32_t* projs, const void* const* d_x,
                                     const void* const* d_W, const lora_segments* seg, void* const* d_out,
                                     void* stream);

/* Whole-model form of lora_layer_forward_group (paper Sec. 2.2: an adapter adds its matrices to the targeted
 * layers of every decoder layer, and the adapter slots hold whole adapters; Sec. 5.1.3: loading time grows with
 * adapter size).  The context was created with n_layers > 1; `layer` (0 .. n_layers - 1) selects which layer's
 * part of every slot the call reads; everything else as lora_layer_forward_group, which is this call with
 * layer 0.  The segment map of one lora_bucket serves every layer of the step.  lora_slots_load enqueues an
 * adapter's copies layer after layer and the forward of a layer waits only for the copies of its own
 * projections, so a step that runs behind a load starts on the first layers while later ones still travel.
 * Errors: as lora_layer_forward_group, INVALID_ARG also for a layer out of range. */
lora_status lora_model_forward_group(lora_ctx *ctx, int32_t layer, int32_t n, const int32_t *projs,
                                     const void *const *d_x, const void *const *d_W, const lora_segments *seg,
                                     void *const *d_out, void *stream);

/* Gate and up of a gated MLP in one call, with their product: d_out[t, n] = silu(gate[t, n]) * up[t, n], where gate
 * and up are the projections proj_gate and proj_up of the same input d_x, each with its adapter term as in
 * lora_layer_forward (paper Sec. 2.2), and silu(z) = z / (1 + exp(-z)).  This is what the `down` projection of the
 * Llama and Qwen2.5 model families reads (the paper's evaluation, Sec. 8.1); formed in the GEMM's epilogue from the
 * fp32 accumulators and rounded to bf16 once, the two projections never travel to memory.  Both projections must
 * have the same d_in and d_out and no bias (lora_set_bias): SHAPE / INVALID_ARG otherwise.  d_out: device bf16
 * [T, d_out].  Always one GEMM launch over full K (plus the shrink launch where it does not ride inside); everything
 * else as lora_layer_forward_group.  Errors: as lora_layer_forward_group. */
lora_status lora_layer_forward_glu(lora_ctx *ctx, int32_t proj_gate, int32_t proj_up, const void *d_x,
                                   const void *d_W_gate, const void *d_W_up, const lora_segments *seg, void *d_out,
                                   void *stream);

/* Whole-model form of lora_layer_forward_glu, as lora_model_forward_group is of lora_layer_forward_group (paper
 * Sec. 2.2: an adapter targets the same projections in every decoder layer): `layer` (0 .. n_layers - 1) selects
 * which layer's part of every slot the call reads; lora_layer_forward_glu is this call with layer 0.  Errors: as
 * lora_layer_forward_glu (the bias rule applies to the projections of that layer), INVALID_ARG also for a layer
 * out of range. */
lora_status lora_model_forward_glu(lora_ctx *ctx, int32_t layer, int32_t proj_gate, int32_t proj_up, const void *d_x,
                                   const void *d_W_gate, const void *d_W_up, const lora_segments *seg, void *d_out,
                                   void *stream);

/* Bias of a backbone projection (paper Sec. 2.2: the adapter's activations are added to the backbone layer's
 * output, which for a layer with a bias is x W^T + b; Sec. 8.1 evaluates on the Qwen2.5 family, whose q, k, v
 * projections have one).  d_bias: device bf16 [d_out_proj], 16-byte aligned, owned by the caller, read by every
 * later lora_layer_forward / lora_layer_forward_group of that projection until it is replaced: it must stay
 * valid and unchanged while such calls may still run.  NULL removes the bias (the state after lora_create).
 * The result becomes bf16(x W^T + b + s (x A^T) B^T): b is added in fp32 before the one rounding.  Host state
 * only: nothing is enqueued and calls already enqueued are not affected.
 * layer: 0 unless the context has n_layers > 1.
 * Errors: INVALID_ARG (layer or proj out of range, misaligned pointer). */
lora_status lora_set_bias(lora_ctx *ctx, int32_t layer, int32_t proj, const void *d_bias);

/* Blocking read-and-clear of the device flag word (synchronises `stream`).  Paper Sec. 2.2: a request is
 * processed only while its adapter resides in GPU memory; a token that violated this was served backbone-only and
 * is reported here.  After LORA_FLAG_INTERNAL the context also sets the counters of the launch back and from then
 * on runs the shrink as a launch of its own (the assumption behind the shrink inside a launch failed once).  Returns
 * LORA_ERR_NOT_RESIDENT if LORA_FLAG_NOT_RESIDENT was set (LORA_ERR_HIP if LORA_FLAG_INTERNAL was), else LORA_OK; *flags (may be NULL)
 * receives the raw word. */
lora_status lora_poll_device_flags(lora_ctx *ctx, uint32_t *flags, void *stream);

/* Slot-table queries (host state, no device access). */
int32_t lora_slot_of(const lora_ctx *ctx, int32_t adapter_id);      /* slot or -1 */
int32_t lora_slot_adapter(const lora_ctx *ctx, int32_t slot);       /* adapter id or -1 */
int32_t lora_slot_first_page(const lora_ctx *ctx, int32_t slot);    /* n_pages > 0: first page of the slot's adapter;
                                                                        -1: empty slot, rank 0, or a context without pages */

/* Kernel-variant selection for experiments and autotuning; value 0 is always the default variant and
 * unknown values fall back to it.  Every variant computes the same result to the same tolerance. */
enum {
    LORA_TUNE_FUSED_VARIANT = 0, /* tile shape / wave layout of the fused GEMM */
    LORA_TUNE_SPLIT_VARIANT = 1, /* tile shape / wave layout of the split-K GEMM */
    LORA_TUNE_COPY_ENGINE = 2,   /* what carries an adapter's matrices into its slot (lora_slots_load) */
    LORA_TUNE_INLINE_SHRINK = 3, /* fused path up to 1024 tokens: shrink by the first workgroups of the GEMM launch */
    LORA_TUNE_SHRINK_WAIT_TEST = 4 /* test aid, value n > 0: in such a launch the tile workgroups expect one report more
                                      than will come and give up after n polls, so that the expired-wait handling
                                      (LORA_FLAG_INTERNAL, counter reset, fallback) can be exercised from the host
                                      with every kernel ending normally; the outputs of that launch are undefined, as after any
                                      expired wait (the tile workgroups may have read shrink results that were not there yet) */
};
/* Values of LORA_TUNE_INLINE_SHRINK. */
enum {
    LORA_INLINE_SHRINK_AUTO = 0, /* when the tiles leave CUs idle and those can finish the shrink in time */
    LORA_INLINE_SHRINK_OFF = 1,  /* always a separate shrink launch */
    LORA_INLINE_SHRINK_ON = 2    /* whenever at least 8 CUs have no tile */
};
/* Values of LORA_TUNE_COPY_ENGINE. */
enum {
    LORA_COPY_AUTO = 0,   /* the copy engine when every contiguous run of the load has at least 128 KiB, else the kernel */
    LORA_COPY_KERNEL = 1, /* a kernel that reads the pinned host memory, a batch of runs per launch */
    LORA_COPY_ENGINE = 2  /* hipMemcpyAsync per run */
};
/* Values of LORA_TUNE_FUSED_VARIANT: tile (rows x columns x K tile), wavefronts per workgroup. */
enum {
    LORA_FUSED_AUTO = 0,
    LORA_FUSED_256x256x32_W4 = 1,
    LORA_FUSED_256x256x32_W4_3STAGES = 2,
    LORA_FUSED_128x128x32_W4 = 3,
    LORA_FUSED_256x128x32_W8 = 4,
    LORA_FUSED_256x128x32_W8_ALLCOPY = 5, /* every wavefront issues tile copies */
    LORA_FUSED_256x128x64_W8 = 8,         /* 64-wide K tiles: whole 128-byte lines per row segment */
    LORA_FUSED_128x128x64_W4 = 9,
    LORA_FUSED_256x256x64_W8 = 10,
    LORA_FUSED_256x192x64_W8 = 11,
    LORA_FUSED_256x256x32_W8 = 12,
    LORA_FUSED_256x128x64_W4 = 13,        /* four wavefronts with 128 x 64 wave tiles: fewer LDS reads per MFMA */
    LORA_FUSED_256x256x64_W4 = 14,
    LORA_FUSED_STAGED_256x256x64_W8 = 15, /* tiles staged through registers (ordinary loads, LDS writes), two LDS stages:
                                             what LORA_FUSED_AUTO takes above 1024 tokens when the grid fills the chip */
    LORA_FUSED_STAGED_256x256x64_W4 = 16
};
/* Values of LORA_TUNE_SPLIT_VARIANT. */
enum {
    LORA_SPLIT_AUTO = 0,
    LORA_SPLIT_256x128x32_W4 = 1,
    LORA_SPLIT_256x64x32_W4 = 2,
    LORA_SPLIT_128x128x32_W4 = 3,
    LORA_SPLIT_128x128x32_W4_8STAGES = 4,
    LORA_SPLIT_256x128x64_W8 = 6,
    LORA_SPLIT_128x128x64_W4 = 7,
    LORA_SPLIT_256x128x32_W8 = 8,
    LORA_SPLIT_256x128x64_W4 = 9
};
lora_status lora_set_tuning(lora_ctx *ctx, int32_t key, int32_t value);

/* Kernel launches made by the most recent lora_layer_forward on this context: fills up to `cap`
 * entries of names[] (static strings) and returns the count.  For benchmarks and profiling. */
int32_t lora_last_launches(const lora_ctx *ctx, const char **names, int32_t cap);

/* Per-kernel timing for benchmarks.  While enabled, every kernel the context launches is
 * bracketed by a pair of HIP timing events on its own stream.  lora_profile_collect waits for the
 * recorded events, adds them to running totals per kernel name and returns the number of distinct
 * names; up to `cap` entries of names[] (valid until lora_profile_reset or lora_destroy),
 * total_ms[] and counts[] are filled.  At most 8192 launches are recorded between two collects. */
lora_status lora_profile_enable(lora_ctx *ctx, int32_t on);
int32_t lora_profile_collect(lora_ctx *ctx, const char **names, double *total_ms, int64_t *counts, int32_t cap);
lora_status lora_profile_reset(lora_ctx *ctx);

/* Ceiling probes for benchmarks (measurement aids, not on the serving path; the paper's latency model, Sec. 5.2,
 * prices a step by what the weight stream and the matrix cores sustain).  Both enqueue one launch on `stream`.
 * lora_calibrate_stream: `workgroups` workgroups of 512 threads read `bytes` of device memory at d_src (16-byte
 * aligned) once, 16 bytes per lane and load, eight loads in flight per lane; d_sink: device, 4 * workgroups bytes
 * (practically never written).  Bytes / launch time = the read rate a plain stream reaches on this machine.
 * lora_calibrate_mfma: `workgroups` workgroups of four wavefronts issue iters * 16 back-to-back bf16 MFMAs
 * (32x32x16, 32768 flop each) per wavefront; d_sink: device, 1024 * workgroups bytes; d_ticks: device,
 * 16 * workgroups bytes: per workgroup the shader clock ticks and the 100 MHz wall clock ticks of its loop, so
 * that the clock the chip sustained under this load can be read off.
 * Errors: INVALID_ARG, HIP. */
lora_status lora_calibrate_stream(const void *d_src, size_t bytes, int32_t workgroups, void *d_sink, void *stream);
lora_status lora_calibrate_mfma(int32_t workgroups, int32_t iters, void *d_sink, void *d_ticks, void *stream);

/* Adapter placement over GPUs (paper Sec. 7, the greedy caching algorithm with its feasibility test).  Host
 * code, no device access.  Input: for each of n_adapters its size (rank, > 0) and Poisson arrival rate
 * (>= 0), and the number of GPUs.  The two predictors are the caller's: given the sizes and rates of all
 * adapters that would share one GPU (n of them, in the order they were taken from the queue) and a configuration
 * a_max, predict_throughput returns the expected throughput (any unit, only compared) and predict_starvation
 * nonzero if requests would starve; `user` is handed through.  Adapters are taken in priority order (largest
 * size first; inside one size by arrival rate alternating high and low; ties by index) and included in the open
 * GPU provisionally; whenever that GPU's adapter count reaches one of 8 16 32 64 96 128 160 192 256 320 384 the
 * provisional set is tested: the GPU's a_max becomes the better of its current value and the next value of that
 * list (the next value outright while it has none), and if starvation is predicted for it the provisional set
 * goes back to the queue and the GPU takes no more adapters.  What is still provisional at the end is tested
 * once more.  Output: gpu_of[a] in [0, n_gpus) for every adapter, a_max_of[g] for every GPU (0: GPU unused).
 * Errors: INVALID_ARG; STARVATION when an adapter finds no GPU left or the last test fails (outputs are then
 * unspecified). */
typedef double (*lora_throughput_fn)(void *user, int32_t n, const int32_t *sizes, const double *rates, int32_t a_max);
typedef int32_t (*lora_starvation_fn)(void *user, int32_t n, const int32_t *sizes, const double *rates, int32_t a_max);
lora_status lora_place_adapters(int32_t n_adapters, const int32_t *size, const double *rate, int32_t n_gpus,
                                lora_throughput_fn predict_throughput, lora_starvation_fn predict_starvation,
                                void *user, int32_t *gpu_of, int32_t *a_max_of);

/* The priority order alone (paper Sec. 7, PrioritySorting): order_out[k] = index of the k-th adapter to place.
 * Errors: INVALID_ARG. */
lora_status lora_priority_sorting(int32_t n_adapters, const int32_t *size, const double *rate, int32_t *order_out);

const char *lora_status_string(lora_status s);

/* Text of the most recent failing HIP runtime call made by this library on the calling thread
 * ("<call>: <hip error string>"), or "" if none failed.  Valid until the next failure. */
const char *lora_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LORA_MI355_H */
