/*
 * liborbit — batched GQA decode attention over a paged KV cache whose (request, layer) blocks
 * are split between HBM and pinned host memory, for one AMD MI355X (gfx950).
 *
 * The calls follow the paper's problem statement (Section 3.3.1): a batch of requests with
 * context lengths, L layers, a binary placement matrix x[r,l] (1 = KV of request r at layer l
 * stays on the GPU, 0 = it is held in host memory and fetched before the layer runs) and a GPU
 * block budget B_GPU bounded by Eq. (1).  The KV manager semantics (block tables, minimal
 * data movement on a new placement, new KV of offloaded layers written straight to the host,
 * a contiguous prefetch buffer) are those of Section 3.2, "KV Manager".
 *
 * Conventions
 *  - Every call returns ORBIT_OK (0) or a negative ORBIT_E_* code; orbit_last_error() gives
 *    the text.  No exception or abort crosses this boundary.
 *  - "device" pointers are HIP device memory; "host" pointers are ordinary host memory unless
 *    "pinned" is stated.  The library never frees or reallocates caller memory.
 *  - All GPU work is enqueued on the two caller-owned streams (the deferred copies of a plan
 *    switch on one stream the library owns) and is asynchronous to the host unless a call says
 *    it synchronises.  One context must be driven by one thread at a time.
 *  - bf16 everywhere for Q, K, V and the output; accumulation is fp32.
 *  - Keep the streams a process actually uses few: HIP maps them onto four hardware queues per
 *    process by default, and a further busy stream that lands on the queue of compute_stream or
 *    copy_stream serialises the host-link copies with the kernels (measured with two extra
 *    streams that had carried a few copies earlier: 211 ms per step instead of 203 ms).
 *
 * KV block ("page") layout, bf16 elements, P = page_tokens = 16, D = head_dim = 128:
 *    page   = [K tile head 0]..[K tile head Hkv-1][V tile head 0]..[V tile head Hkv-1]
 *    K tile : (tok, dim) at (dim/8)*(P*8) + tok*8 + dim%8
 *    V tile : (tok, dim) at ((((dim/32)*(P/4) + tok/4)*16 + dim%16)*2 + (dim/16)%2)*4 + tok%4
 * (each tile is 4 KiB; a page is Hkv*8 KiB).  Host-resident (request, layer) blocks use the
 * same page layout in one contiguous run of pages.
 */
#ifndef ORBIT_H_
#define ORBIT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORBIT_API __attribute__((visibility("default")))

#define ORBIT_OK               0
#define ORBIT_E_INVAL         -1  /* bad argument                                              */
#define ORBIT_E_CAPACITY      -2  /* Eq. (1) violated: the planner's "infeasible"              */
#define ORBIT_E_HOST_CAPACITY -3  /* pinned host arena too small                               */
#define ORBIT_E_NOT_FOUND     -4  /* unknown request id                                        */
#define ORBIT_E_STATE         -5  /* call not valid now (no plan, window expired, ...)         */
#define ORBIT_E_HIP           -6  /* a HIP runtime call failed                                 */
#define ORBIT_E_NOMEM         -7  /* a host allocation failed; the call changed nothing it can
                                     undo, but the context should be destroyed                 */

#define ORBIT_MAX_LAYERS   128
#define ORBIT_MAX_REQUESTS 256
#define ORBIT_STATIC_SCRATCH_BYTES (16 << 20)  /* split-K scratch of orbit_decode_attention_static, per GPU */

/* flags */
#define ORBIT_FLAG_HOST_ONLY 1    /* run only the host logic (tables, schedules); no GPU call is
                                     made and the arenas may be NULL.  For CPU-side tests.      */
#define ORBIT_FLAG_POISON_STAGING 4 /* debugging aid: once a layer's attention has read its staging range, the
                                     range is overwritten with NaN bit patterns, so that any later read of
                                     stale staged KV (a missing wait, a range reused too early) shows up as
                                     NaN outputs instead of plausible numbers.  Costs one fill per streamed
                                     layer; results are otherwise bit-identical.                           */
#define ORBIT_FLAG_ZERO_COPY 2    /* no staging region and no host->staging copies: the attention
                                     kernel reads offloaded blocks straight from the mapped pinned
                                     host arena over the link.  Eq. (1) then charges no B_buf,
                                     orbit_kv_prefetch is a no-op and prefetch_slots is ignored.
                                     Same arithmetic in the same order as the staged mode, so the
                                     outputs are bit-identical to it.  A measured alternative to
                                     the paper's prefetch buffer (Section 3.3.1), not its method. */

typedef struct orbit_ctx orbit_ctx;

typedef struct {
  int32_t n_layers;               /* L, 1..ORBIT_MAX_LAYERS                                    */
  int32_t n_q_heads;              /* Hq                                                         */
  int32_t n_kv_heads;             /* Hkv; Hq % Hkv == 0 and Hq/Hkv <= 16                        */
  int32_t head_dim;               /* must be 128                                                */
  int32_t page_tokens;            /* must be 16 (16-token KV blocks, Section 2.3)               */
  int32_t max_requests;           /* 1..ORBIT_MAX_REQUESTS                                      */
  int64_t max_tokens_per_request; /* upper bound of any request's length                        */
  float   softmax_scale;          /* <= 0 selects 1/sqrt(head_dim)                              */
  int32_t prefetch_slots;         /* k >= 1: staging region = k * B_buf blocks; 1 = the paper's
                                     single prefetch buffer of Eq. (1)                          */
  int32_t chunk_tokens;           /* tokens per attention work segment (multiple of 32); 0 lets
                                     every launch choose (see orbit_get_work_items)             */
  int32_t decode_window;          /* Delta >= 0: tokens each request may grow under one plan
                                     (the decode window of Section 3.3.1); Eq. (1) is checked
                                     with b_r = ceil((ctx_len + Delta)/16)                      */
  int32_t flags;                  /* ORBIT_FLAG_*                                               */
  void   *hbm_arena;              /* device, caller-owned, 256-byte aligned                     */
  int64_t hbm_arena_bytes;
  void   *host_arena;             /* pinned host (hipHostMalloc / torch pin_memory), caller-owned */
  int64_t host_arena_bytes;
  void   *compute_stream;         /* hipStream_t, caller-owned                                  */
  void   *copy_stream;            /* hipStream_t, caller-owned, must differ from compute_stream */
} orbit_config;

/* Filled by orbit_step when requested; times in milliseconds from HIP events. */
typedef struct {
  float   step_ms;                       /* first enqueue to last kernel on compute_stream     */
  float   attn_ms_total;                 /* sum of attn_ms                                      */
  float   copy_ms_total;                 /* sum of copy_ms                                      */
  float   stall_ms_total;                /* compute_stream time spent waiting for prefetches    */
  int64_t hbm_kv_bytes;                  /* KV bytes attended from resident blocks (and from blocks
                                            still read in place after a plan switch)            */
  int64_t link_kv_bytes;                 /* KV bytes moved host -> staging this step (zero-copy
                                            mode: read over the link by the attention kernel)   */
  int64_t hbm_blocks_reserved;           /* resident blocks + staging region (left of Eq. (1))  */
  int64_t hbm_blocks_budget;             /* B_GPU                                               */
  float   attn_ms[ORBIT_MAX_LAYERS];     /* the layer's attention launch (the step's append is part of it) */
  float   combine_ms[ORBIT_MAX_LAYERS];  /* cross-chunk combine launch, per layer                */
  float   copy_ms[ORBIT_MAX_LAYERS];     /* host -> staging copies of that layer                */
  float   stall_ms[ORBIT_MAX_LAYERS];
  int64_t link_bytes[ORBIT_MAX_LAYERS];
} orbit_step_stats;

/* Static description of the installed plan (host integers). */
typedef struct {
  int64_t page_bytes;
  int64_t budget_blocks;          /* B_GPU                                                      */
  int64_t resident_blocks;        /* sum_r sum_l b_r x[r,l]                                     */
  int64_t buffer_blocks;          /* B_buf = max_l sum_r (1 - x[r,l]) b_r                       */
  int64_t staging_first_page;     /* the staging region is [first, first + staging_blocks)      */
  int64_t staging_blocks;         /* prefetch_slots * B_buf                                     */
  int64_t host_blocks;            /* blocks held in the pinned host arena                       */
  int64_t moved_to_host_blocks;   /* data movement of the last orbit_plan_load (Section 3.2:    */
  int64_t moved_to_hbm_blocks;    /*   only the delta between the two layouts is moved)         */
  int64_t relocated_blocks;       /* resident blocks moved out of the new staging region        */
  int32_t n_requests;
  int32_t chunk_tokens;
  int64_t evicted_blocks;         /* HBM blocks of paused requests the last plan load pushed to host */
  int64_t paused_resident_blocks; /* HBM blocks still held by paused requests (reclaimable)     */
  int32_t paused_requests;
  int32_t reserved_;
  int64_t deferred_to_host_blocks;/* of the blocks the last plan load moved or evicted to the host: those whose
                                     copy runs beside the following steps instead of in front of them      */
  int64_t in_place_blocks;        /* blocks of active requests that the last plan load demoted and that are read
                                     where they were in HBM until their copies have landed                 */
  int64_t reclaimed_blocks;       /* blocks the last plan load wanted in HBM that were still being read in place
                                     there: they took their pages back, nothing was copied (not counted in
                                     moved_to_hbm_blocks)                                                   */
  int64_t still_in_place_blocks;  /* blocks that an earlier plan load demoted, that were still read in place when the
                                     last one came and that go on being read in place under it (they stay offloaded
                                     and it left their old pages alone)                                      */
  int64_t waited_for_deferred;    /* 1 if the last plan load made its copies wait for deferred copies of earlier plan
                                     loads (it touched a page one of them reads or writes), 0 if it ran beside
                                     them or none were outstanding                                           */
} orbit_plan_info;

/* ---- lifetime (ancillary) ------------------------------------------------------------------ */

/* Creates a context, with the GPU it is to run on current.  Allocates the library's own device tables (page
 * table, work list, split partials), one stream of default priority for the deferred copies of a plan switch,
 * and reserves the host-side storage its calls need.  Fails with ORBIT_E_INVAL on an unsupported shape. */
ORBIT_API int orbit_create(const orbit_config *cfg, orbit_ctx **out);
/* Synchronises both streams, frees the library's own memory.  Caller arenas are untouched. */
ORBIT_API int orbit_destroy(orbit_ctx *ctx);
/* Text of the last error on this context (or of the last failed orbit_create if ctx is NULL). */
ORBIT_API const char *orbit_last_error(orbit_ctx *ctx);

/* ---- a1: plan install (Section 3.3.1: x[r,l], b_r, Eq. (1); Section 3.2: KV Manager) -------- */

/* Pure function, no context: evaluates Eq. (1) for a placement.
 * placement_bitmap: host, row-major [n_req][ceil(L/8)], bit l (LSB first) = x[r,l].
 * out4 (host): {resident blocks, B_buf, resident + prefetch_slots*B_buf, host blocks};
 * prefetch_slots >= 0 (0 = the zero-copy mode, which has no staging region). */
ORBIT_API int orbit_plan_check(int32_t n_req, int32_t n_layers, int32_t page_tokens, const int32_t *ctx_len,
                     const uint8_t *placement_bitmap, int32_t prefetch_slots, int32_t decode_window,
                     int64_t *out4);

/* Installs a placement for the batch {req_ids}.  All pointers are host memory.
 *   req_ids[n_req]  distinct ids; active ids not listed are dropped and their blocks freed
 *                   (paused ones stay paused); ids not known yet are created holding ctx_len
 *                   tokens of undefined content (write them with orbit_kv_fill).
 *   ctx_len[n_req]  tokens held now; for a known request it must equal its current length.
 *   placement_bitmap as in orbit_plan_check.
 *   hbm_budget_bytes  B_GPU = floor(min(budget, arena) / page bytes).
 * Checks Eq. (1) (ORBIT_E_CAPACITY) and the host arena (ORBIT_E_HOST_CAPACITY); on any error
 * NOTHING changes.  On success it moves only the blocks whose tier changed, plus resident
 * blocks that sit where the new contiguous staging region goes, and rebuilds the tables.
 * The host does not wait for the GPU (no stream or device synchronisation, as Section 4 asks):
 * the migrations the new plan needs at once are enqueued on copy_stream behind everything already
 * enqueued on compute_stream, and compute_stream waits for them before any later call's work.
 * Blocks that leave HBM without their pages being needed at once (orbit_plan_info.deferred_to_host_blocks)
 * are copied out on a stream of the library's own, beside the following steps.  Until a layer's copies have
 * landed, attention reads such blocks of active requests where they were (orbit_plan_info.in_place_blocks:
 * their old pages are not handed out before a later plan load), a step's new token is written there and into
 * the host run, and the layer is not prefetched for them; the first prefetch of the layer issued after its
 * copies have completed (in the zero-copy mode: the first attention call) switches them to the staging region
 * (to their host pages).  Calls that need the host copy itself (orbit_kv_fill, orbit_kv_read, orbit_kv_append, a
 * decode window that outgrows the old pages) wait for the copies stream-side.  Under the next plan load a block that
 * is still read in place and stays offloaded goes on being read in place if its old pages are not needed
 * (orbit_plan_info.still_in_place_blocks); one that the plan wants in HBM again keeps the pages it is being read from
 * and nothing is copied (orbit_plan_info.reclaimed_blocks); any other is read from its host run once its layer's
 * copies have landed.  The plan load
 * waits for the copies itself only if it hands out an HBM page one of them still reads or a host page one of them
 * still writes, or moves a block whose host run they are still filling (orbit_plan_info.waited_for_deferred).
 * ORBIT_E_STATE if a prefetched layer has not been attended yet. */
ORBIT_API int orbit_plan_load(orbit_ctx *ctx, int32_t n_req, const int64_t *req_ids, const int32_t *ctx_len,
                    const uint8_t *placement_bitmap, int64_t hbm_budget_bytes);

ORBIT_API int orbit_get_plan_info(orbit_ctx *ctx, orbit_plan_info *out);

/* Pause-Resume (Section 3.4) with the removable cache of Section 4.  orbit_request_pause takes an
 * active request out of the batch (the other requests keep their placement; tables are rebuilt,
 * stream-ordered like orbit_plan_load) but leaves its KV where it is.  Its HBM blocks no
 * longer count against Eq. (1): a later orbit_plan_load that needs the room evicts them to the
 * host arena one layer at a time, only as many as needed.  A paused request is resumed by
 * listing it in orbit_plan_load again (only layers that were evicted and are wanted in HBM move
 * back), and forgotten with orbit_request_drop. */
ORBIT_API int orbit_request_pause(orbit_ctx *ctx, int64_t req_id);
ORBIT_API int orbit_request_drop(orbit_ctx *ctx, int64_t req_id);

/* ---- a3: KV writes (Section 2.3 block growth; Section 3.2 direct-to-host writes) ------------ */

/* Bulk write (the product of prefill): tokens [first_token, first_token + n_tokens) of
 * (req_id, layer), k and v device pointers, token-major [n_tokens][Hkv][D] bf16, read
 * asynchronously on compute_stream.  The range must lie inside the request's current length. */
ORBIT_API int orbit_kv_fill(orbit_ctx *ctx, int64_t req_id, int32_t layer, int64_t first_token,
                  int64_t n_tokens, const void *k, const void *v);

/* Gather back to token-major (diagnostic; bit-exact inverse of orbit_kv_fill/append).
 * k_out, v_out: device [n_tokens][Hkv][D] bf16.  Asynchronous on compute_stream. */
ORBIT_API int orbit_kv_read(orbit_ctx *ctx, int64_t req_id, int32_t layer, int64_t first_token,
                  int64_t n_tokens, void *k_out, void *v_out);

/* Appends ONE token to (req_id, layer): k, v device [Hkv][D] bf16, read asynchronously on
 * compute_stream.  A new block is started only when the length is a multiple of 16; it comes
 * from the blocks the plan reserved (ORBIT_E_STATE once the decode window is used up).  For an
 * offloaded layer the token is written straight to its host slot, and also into the staging
 * copy if that layer is currently prefetched (compute_stream first waits, stream-side, for that
 * copy to land, so the transfer cannot overwrite the token).  Lengths are kept per (request, layer). */
ORBIT_API int orbit_kv_append(orbit_ctx *ctx, int64_t req_id, int32_t layer, const void *k, const void *v);

/* The same for every request of the plan at once (what a model's layer does during decode):
 * k, v device [n_req][Hkv][D] bf16 in plan order, one launch per 64 requests.  All or nothing:
 * ORBIT_E_STATE, with no length changed, if any request has used up its decode window. */
ORBIT_API int orbit_kv_append_batch(orbit_ctx *ctx, int32_t layer, const void *k, const void *v);

/* ---- a4/a5: prefetch and gating (Section 3.3.1, "Scheduling KV Prefetching") ---------------- */

/* Enqueues, on copy_stream, the host -> staging copies of every offloaded request of `layer`
 * (smallest first) and records that layer's "ready" event.  A staging range is reused only
 * after the layer that read it has been enqueued and has finished (stream-side wait, never a
 * host wait).  No-op for a layer with nothing offloaded or already prefetched.
 * ORBIT_E_STATE if the range is still needed by a prefetched layer not yet attended. */
ORBIT_API int orbit_kv_prefetch(orbit_ctx *ctx, int32_t layer);

/* ---- a6/a7: attention (Section 2.1 and Fig. 1: decode reads the KV of every earlier token and
 *      computes one token; grouped-query attention shares a KV head among a group of query heads) ---- */

/* Batched decode attention of one layer over the stored lengths of that layer.
 * q: device [n_req][Hq][D] bf16 in plan order; out: device [n_req][Hq][D] bf16;
 * out_f32: optional device [n_req][Hq][D] fp32 (same values before the bf16 rounding), or NULL.
 * Prefetches the layer if needed, waits for it stream-side, runs split-K attention and the
 * combine on compute_stream.  ORBIT_E_INVAL if any request of the plan holds no token. */
ORBIT_API int orbit_decode_attention(orbit_ctx *ctx, int32_t layer, const void *q, void *out, float *out_f32);

/* One layer of a decode step, as a model's layer calls it between its QKV projection and its output projection
 * (Section 3, "Runtime Executor": layers run in order; Section 3.2: the new KV of an offloaded layer goes straight
 * to the host): appends k_new, v_new (device [n_req][Hkv][D] bf16, plan order) to every request of `layer` and
 * attends q over the grown cache, in ONE launch (the workgroup that owns the new token's position takes its row
 * from k_new / v_new, attends to it and stores it into the resident page, or into the staging copy and the host
 * run), where orbit_kv_append_batch + orbit_decode_attention take two and a separate pass over the token.  Results
 * equal those of the two calls, and of orbit_step, bit for bit.  Prefetches the layer if needed (over the lengths
 * before the new token); to run ahead, call orbit_kv_prefetch for this layer and then for the following ones
 * before the call (in that order: a later layer may be given the staging range this one needs).  q, out, out_f32 as
 * for orbit_decode_attention.  ORBIT_E_STATE, with no length changed, if any request has used up its decode window
 * or the layer's staging range is still needed by a prefetched layer not yet attended. */
ORBIT_API int orbit_decode_layer(orbit_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                 void *out, float *out_f32);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same work, same results (bit for bit) and same errors as
 * orbit_decode_attention, but the call allocates nothing (no device memory, no pinned memory; the
 * host-side storage it uses was reserved by orbit_create): the split-K partial results live in a static device array of
 * ORBIT_STATIC_SCRATCH_BYTES that is part of the library's image on every GPU the library runs on
 * (held until the process ends) instead of the context's own buffers.
 * ORBIT_E_CAPACITY, with nothing enqueued, if the batch needs more: S * Hkv partial slots of
 * (Hq/Hkv * 128 + 32) * 4 bytes, S = the number of work segments (see orbit_get_work_items; with
 * chunk_tokens 0 the 70B workload at batch 32 needs 620 segments = 21 MB and does not fit, the 8B
 * workloads of up to 64 requests do).
 * The array is shared by every context and every call on that GPU and keeps the last call's
 * contents (nothing in it needs clearing: every partial is written before it is read).  Calls that overlap on one
 * GPU (two streams, two contexts, two threads) race on it: serialise them.  The context must have
 * been created with its GPU current. */
ORBIT_API int orbit_decode_attention_static(orbit_ctx *ctx, int32_t layer, const void *q, void *out, float *out_f32);

/* ---- a8: one decode step (Section 3, "Runtime Executor": layers run in order, prefetches of
 *      offloaded layers run ahead, compute / transfer time and memory in use are recorded) ---------- */

/* For l = 0..L-1 in order: append k_new[l], v_new[l] to every request, then attend q[l] over
 * the grown cache into out[l]; prefetches run ahead on copy_stream.
 * q, out: device [L][n_req][Hq][D] bf16; k_new, v_new: device [L][n_req][Hkv][D] bf16.
 * stats: NULL, or host memory to fill; filling it blocks until the step has finished.
 * The call only enqueues work.  Keep the host within a few steps of the GPU (a serving loop that
 * samples a token per step does so by itself): with dozens of steps queued, the HIP runtime's
 * queues fill up and throughput drops by several percent (measured: 100 steps run ahead freely
 * took 6.5 % longer per step than with at most two outstanding).
 * ORBIT_E_STATE (no plan, an empty plan, decode window used up, a prefetched layer left
 * unattended) and ORBIT_E_INVAL (NULL pointer) are detected before anything is enqueued and
 * change nothing.  ORBIT_E_HIP can strike mid-step: the layers already enqueued keep their
 * appended token, so the context is then only good for orbit_destroy. */
ORBIT_API int orbit_step(orbit_ctx *ctx, const void *q, const void *k_new, const void *v_new, void *out,
               orbit_step_stats *stats);

/* ---- planner helpers (host only, no context, no GPU) ---------------------------------------- */

/* Distance-driven candidates of Section 3.3.2: writes the distinct values of floor(L/k),
 * k = 2..L, in descending order (16 10 8 6 5 4 3 2 1 for L = 32) and returns their number D(L)
 * (<= 2*floor(sqrt(L)) - 1), or a negative error.  counts_out may be NULL. */
ORBIT_API int orbit_distance_options(int32_t n_layers, int32_t *counts_out, int32_t cap);

/* One request's placement row for an offload count: every N-th layer (1-based l with l % N == 0)
 * is offloaded, N the largest distance with floor(L/N) == count; 0 keeps all layers on the GPU,
 * L offloads all.  row_out: ceil(L/8) bytes, bit l LSB-first, 1 = GPU. */
ORBIT_API int orbit_distance_pattern(int32_t n_layers, int32_t offload_count, uint8_t *row_out);

/* Modelled decode latency of a placement (Section 3.3.1, the prefetch rules behind Algorithm 1,
 * run as an event-driven simulation with even bandwidth sharing).  blocks[r] = b_r,
 * blocks_per_time = link bandwidth B in blocks per time unit, comp[l] = compute time of layer l.
 * stall_out (optional, L doubles) receives the stall time in front of each layer; *t_batch the
 * total (sum comp + sum stall).  All pointers host memory. */
ORBIT_API int orbit_model_latency(int32_t n_req, int32_t n_layers, const int64_t *blocks,
                                  const uint8_t *placement_bitmap, double blocks_per_time, const double *comp,
                                  double *stall_out, double *t_batch);

/* Searches the pruned space (per request: keep all, the D(L) distance-driven counts, offload all)
 * for the placement of minimum modelled latency that satisfies Eq. (1) with gpu_blocks and
 * prefetch_slots.  Exhaustive if the space has at most max_evals points (ties: fewest offloads
 * for the earliest request); otherwise coordinate descent from the best uniform plan, which stops
 * with the best plan found so far once max_evals placements have been simulated (the uniform
 * plans, one per candidate count, are always tried, so *evals_out <= max(max_evals, D(L) + 2)).
 * bitmap_out: [n_req][ceil(L/8)].  Returns ORBIT_E_CAPACITY if nothing is feasible (the
 * planner's "infeasible", after which the paper pauses a request). */
ORBIT_API int orbit_plan_search(int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks,
                                int32_t prefetch_slots, double blocks_per_time, const double *comp,
                                int64_t max_evals, uint8_t *bitmap_out, double *t_batch, int64_t *evals_out);

#define ORBIT_SEARCH_STAGGER 1    /* flag of orbit_plan_search_or_pause and orbit_planner_submit: search the
                                     staggered space of orbit_plan_search_staggered                */

/* The same search over a wider space of our own: request r (plan order) takes its distance-driven
 * pattern rotated right by r layers.  Counts and distances are the paper's; the rotation keeps
 * requests from offloading the same layers, which shrinks B_buf in Eq. (1) and evens out the
 * link load.  Same arguments, results and errors as orbit_plan_search. */
ORBIT_API int orbit_plan_search_staggered(int32_t n_req, int32_t n_layers, const int64_t *blocks, int64_t gpu_blocks,
                                          int32_t prefetch_slots, double blocks_per_time, const double *comp,
                                          int64_t max_evals, uint8_t *bitmap_out, double *t_batch,
                                          int64_t *evals_out);

/* Pause-Resume fallback (Section 3.4) in its capacity form: when no placement of the batch
 * satisfies Eq. (1), the request with the largest sum of KV blocks and deposited tokens is
 * paused (ties: the later request) and the search runs again on the rest, until a plan exists.
 * deposited_tokens[r] >= 0: tokens waiting in request r's Token-Deposit.  flags: 0 or
 * ORBIT_SEARCH_STAGGER.  paused_out[r] = 1 marks the victims (hand them to orbit_request_pause and
 * leave them out of orbit_plan_load); bitmap_out keeps one row per original request (rows of
 * paused requests are all ones and unused).  Returns the number of paused requests (0 = the whole
 * batch fits) or a negative error; never ORBIT_E_CAPACITY, since an empty batch always fits. */
ORBIT_API int orbit_plan_search_or_pause(int32_t n_req, int32_t n_layers, const int64_t *blocks,
                                         const int64_t *deposited_tokens, int64_t gpu_blocks, int32_t prefetch_slots,
                                         double blocks_per_time, const double *comp, int64_t max_evals, int32_t flags,
                                         uint8_t *bitmap_out, uint8_t *paused_out, double *t_batch);

/* Background planner (Section 4: the planner runs in its own thread and solves one decode
 * iteration ahead; the executor collects the finished plan in the next iteration and hands it to
 * orbit_plan_load).  One worker thread per handle.  orbit_planner_submit copies its arguments
 * (same meaning as orbit_plan_search; flags: 0 or ORBIT_SEARCH_STAGGER) and returns a ticket > 0 at once; a submission replaces
 * one that has not started yet.  orbit_planner_poll delivers the newest finished plan not yet
 * collected: returns 1 and fills ticket_out / bitmap_out ([n_req][ceil(L/8)], bitmap_cap bytes
 * available) / t_batch / evals_out, 0 if none is ready, ORBIT_E_CAPACITY if that job found
 * nothing feasible (ticket_out still set), ORBIT_E_INVAL if bitmap_cap is too small (the plan
 * stays collectable).  wait != 0 blocks until every submitted job has finished.
 * orbit_planner_destroy joins the thread.  Calls on one handle must come from one thread. */
typedef struct orbit_planner orbit_planner;
ORBIT_API int orbit_planner_create(orbit_planner **out);
ORBIT_API int orbit_planner_destroy(orbit_planner *p);
ORBIT_API int64_t orbit_planner_submit(orbit_planner *p, int32_t n_req, int32_t n_layers, const int64_t *blocks,
                                       int64_t gpu_blocks, int32_t prefetch_slots, double blocks_per_time,
                                       const double *comp, int64_t max_evals, int32_t flags);
ORBIT_API int orbit_planner_poll(orbit_planner *p, int32_t wait, int64_t *ticket_out, uint8_t *bitmap_out,
                                 int64_t bitmap_cap, double *t_batch, int64_t *evals_out);

/* ---- Token-Deposit and profile refresh (host only; Section 3.2 and Section 3.4) --------------- */

typedef struct orbit_deposit orbit_deposit;

/* One request's deposit: a FIFO of 4-byte token ids released at the SLO rate.  Times are doubles
 * in any unit; slo_interval > 0 in the same unit. */
ORBIT_API int orbit_deposit_create(double slo_interval, orbit_deposit **out);
ORBIT_API int orbit_deposit_destroy(orbit_deposit *d);
/* A token was generated at time `now` (non-decreasing across calls). */
ORBIT_API int orbit_deposit_push(orbit_deposit *d, int32_t token, double now);
/* The request finished at `now`: whatever is still deposited becomes due at once. */
ORBIT_API int orbit_deposit_finish(orbit_deposit *d, double now);
/* Delivers, in order, every token due by `now`: one per SLO interval while tokens are deposited,
 * immediately on generation when the deposit was empty.  Writes up to cap tokens and their
 * delivery times (the instant each became due, not `now`); returns how many, or a negative error. */
ORBIT_API int64_t orbit_deposit_release(orbit_deposit *d, double now, int32_t *tokens_out, double *times_out,
                                        int64_t cap);
/* out4: {tokens waiting, tokens delivered, user-visible interval violations, largest size seen}. */
ORBIT_API int orbit_deposit_stats(orbit_deposit *d, int64_t *out4);

/* SLO accounting of one request over a run of decode steps (the metrics of Section 2.1 behind the
 * Token-Deposit of Section 3.2).  step_latency[k] >= 0 is the duration of step k, which ends with one
 * new token; the clock starts at the instant the request's previous token was delivered, with an
 * empty deposit.  A time between tokens above slo_interval is a TBT violation: counted on generation
 * times (backend_violations: what the engine did) and on delivery times behind the deposit
 * (visible_violations: what the user sees; never more than the former).  tpot = run time / tokens,
 * tpot_violated = it exceeds the same target.  max_deposit = most tokens waiting at a generation
 * instant.  finish_at_end != 0: the request finishes with the last step and what is still deposited
 * leaves in one burst.  All pointers host memory. */
typedef struct {
  int64_t tokens, backend_violations, visible_violations, max_deposit;
  double  tpot, max_visible_gap;
  int32_t tpot_violated, reserved_;
} orbit_slo_report;
ORBIT_API int orbit_slo_replay(const double *step_latency, int64_t n_steps, double slo_interval, int32_t finish_at_end,
                               orbit_slo_report *out);

/* Profile-mismatch trigger: returns 1 if |predicted - observed| > fraction * predicted, else 0. */
ORBIT_API int orbit_profile_mismatch(double predicted, double observed, double fraction);
/* profile[i] <- (1 - weight) * profile[i] + weight * observed[i], 0 <= weight <= 1. */
ORBIT_API int orbit_profile_ewma(double *profile, const double *observed, int64_t n, double weight);

/* ---- host-side introspection (integers only; used by tests) --------------------------------- */

/* Page ids that attention reads for (req_id, layer): arena ids for a resident block list,
 * staging-region ids for an offloaded one.  Writes up to cap ids, returns the reserved count
 * (or a negative error).  tier: 1 = HBM, 0 = host, 2 = host but still read in place from the HBM
 * pages it had (then those pages are listed); host_first_page: index of the run's first
 * page in the host arena (or -1); length: tokens stored. */
ORBIT_API int64_t orbit_get_pages(orbit_ctx *ctx, int64_t req_id, int32_t layer, int32_t *tier,
                        int64_t *host_first_page, int32_t *length, int32_t *pages_out, int64_t cap);

/* Attention work segments of `layer` for the current lengths: rows {request index, first token,
 * tokens, position in the launch order}, by request and first token.  Every request is cut into chunks
 * of C tokens, C = chunk_tokens if the context fixed it, else the largest power of two in [128, 4096]
 * that still gives every compute unit a workgroup (requests are not cut when none is longer than 512
 * tokens, or when none is longer than 4096 and whole requests already fill half of the units); longest
 * segments are launched first.  A request cut into
 * several segments is merged by the combine launch in token order.  Returns the segment count. */
ORBIT_API int64_t orbit_get_work_items(orbit_ctx *ctx, int32_t layer, int32_t *items_out, int64_t cap);

/* Copy schedule of the installed plan: rows {layer, request index, staging first page,
 * reserved pages, position of the layer's range in the staging region}, in issue order.
 * Returns the row count. */
ORBIT_API int64_t orbit_get_copy_schedule(orbit_ctx *ctx, int32_t *rows_out, int64_t cap);

#ifdef __cplusplus
}
#endif
#endif /* ORBIT_H_ */
