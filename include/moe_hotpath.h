/*
 * moe_hotpath.h -- C ABI of the MI355X (gfx950) MoE-layer hot path.
 *
 * One MoE block as the paper's Section 2.1 states it: the gate computes routing
 * weights with a softmax and selects the top-k experts of every token, and the
 * block output is the weighted sum of those experts' outputs,
 *
 *        e_j, w_j = Gate(a)          x' = sum_{j<k} w_j * Expert_{e_j}(a).
 *
 * An expert is the three linear maps gate_proj, up_proj, down_proj
 * (Section 4.4) used as a SiLU-gated FFN.  Experts that are not resident in
 * device memory are streamed from pinned host memory into fixed, pre-registered
 * device slots on a side stream (Section 4.4: an on-demand double buffer plus a
 * prefetch buffer in two groups, current layer / next layer) while the
 * resident experts compute.  Where an expert's bytes come from never changes
 * the result.
 *
 * Conventions
 * -----------
 *  - All pointers are DEVICE pointers unless the parameter name starts with
 *    `host_` or the comment says "host".  The caller owns every buffer it
 *    passes; the library owns only what moe_create() allocates.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Hot calls enqueue work on it and return; they never allocate device
 *    memory.  Results are valid once the stream has been synchronised.
 *  - Storage dtype MOE_BF16: X, Wr and expert matrices are bfloat16, products
 *    are accumulated in float32 (router: float64), `out` is bfloat16.
 *    MOE_F32: everything float32 (router accumulates in float64).
 *  - X [T,H] and Wr [E,H] are row-major.  Wg, Wu [F,H] and Wd [H,F] are
 *    row-major or tiled, see moe_weight_layout.
 *  - A = T*k routed assignments, flat id i = t*k + j.  Shared experts (S of
 *    them) see every token with weight one and are not part of the gate.
 *  - Every entry point returns MOE_OK or a negative moe_status; nothing throws
 *    or aborts across this boundary.  moe_last_error() gives the reason.
 *  - Same inputs give bit-identical outputs from run to run, and outputs do
 *    not depend on residency or prefetch masks.
 *
 * Limits: 1 <= k <= E <= 128; k <= 16; S <= 8; H and F multiples of 128
 * (MOE_BF16) or of 8 (MOE_F32); T*(k+S) < 2^24.
 */
#ifndef MOE_HOTPATH_H
#define MOE_HOTPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,   /* NULL pointer, shape outside the limits, ...  */
  MOE_ERR_UNSUPPORTED = -2,   /* legal request this build cannot serve       */
  MOE_ERR_WORKSPACE = -3,     /* workspace missing or too small              */
  MOE_ERR_HIP = -4,           /* a HIP runtime call failed                   */
  MOE_ERR_SLOT_EXHAUSTED = -5 /* no streaming slot can hold the request      */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/* Memory layout of the expert matrices (the paper fixes none; Section 4.4 only
 * names gate_proj, up_proj, down_proj).
 * MOE_ROW_MAJOR: Wg, Wu [F,H] and Wd [H,F] row-major.
 * MOE_TILED (MOE_BF16 only): every 16-row x 32-column block of a matrix
 *   [N,K] is one contiguous KiB -- block (n16, ks) at element offset
 *   (n16*(K/32) + ks)*512; inside it lane l = r + 16 g holds
 *   W[16 n16 + r][32 ks + 8 g .. 8 g + 7] at element offset 8 l.  That is the
 *   register image of the matrix-core operand, so a wavefront reads 1 KiB in a
 *   row per load instead of 16 rows x 64 bytes.  moe_pack_weights() converts;
 *   it is meant to run once, when an expert is loaded.  Same size in bytes, so
 *   slots, host copies and transfers are unaffected. */
typedef enum { MOE_ROW_MAJOR = 0, MOE_TILED = 1 } moe_weight_layout;

/* Problem shape of one call.  T may change from call to call. */
typedef struct {
  int32_t T;      /* tokens                               */
  int32_t H;      /* hidden size                          */
  int32_t E;      /* routed experts                       */
  int32_t k;      /* experts per token                    */
  int32_t F;      /* expert FFN width                     */
  int32_t S;      /* shared (always-on) experts           */
  int32_t dtype;  /* moe_dtype                            */
  int32_t weight_layout; /* moe_weight_layout of Wg, Wu, Wd (not of Wr, X) */
} moe_shape;

/* The three matrices of one expert (Section 4.4). */
typedef struct {
  const void* Wg; /* gate_proj [F,H] */
  const void* Wu; /* up_proj   [F,H] */
  const void* Wd; /* down_proj [H,F] */
} moe_expert_ptrs;

typedef struct moe_ctx moe_ctx;

/* Library version string (static storage). */
const char* moe_version(void);

/* Reason of the calling thread's most recent failure (static/thread-local
 * storage, valid until that thread's next failing call). */
const char* moe_last_error(void);

/* Bytes of device workspace that moe_layer_forward() (and therefore any single
 * hot call) needs for `shape`.  Returns 0 if the shape is invalid.  The caller
 * allocates it once (256-byte aligned) and passes it to the hot calls. */
size_t moe_workspace_bytes(const moe_shape* shape);

/* ---- a1 + a2: router GEMM, softmax, top-k, renormalised weights ----------
 * Section 2.1 "Gate(a)".  logit[t,e] = bias[e] + sum_h X[t,h]*Wr[e,h],
 * accumulated in float64 so that the selection matches a float64 reference
 * bit for bit whenever neighbouring logits differ by more than ~1e-12.
 * k rounds of arg-max over the logits, ties to the lowest expert index;
 * topk_idx[t,:] is in order of selection (descending logit).
 * topk_w[t,j] = softmax(logit[t,:])[e_j] / sum_j' softmax(logit[t,:])[e_j'].
 *   X [T,H], Wr [E,H]  storage dtype;  bias [E] float32 or NULL (= zeros)
 *   topk_idx [T,k] int32, topk_w [T,k] float32          (outputs)
 *   logits_out [T,E] float64 or NULL                      (optional output)
 *   workspace  moe_workspace_bytes(shape) bytes; may be NULL when logits_out
 *              is given (the logits need a home between the two kernels)
 * T == 0 is legal and does nothing.  MOE_ERR_WORKSPACE when both logits_out
 * and workspace are NULL. */
moe_status moe_route(const moe_shape* shape, const void* X, const void* Wr,
                     const float* bias, int32_t* topk_idx, float* topk_w,
                     double* logits_out, void* workspace, void* stream);

/* ---- a3: bucket the assignments by expert --------------------------------
 * The per-expert pending-token counts of Section 4.3.2 (Premise 1) plus the
 * permutation the grouped FFN consumes.  Stable: inside an expert's bucket the
 * flat assignment ids ascend.
 *   topk_idx [T,k] int32 (values in [0,E))
 *   count [E], offset [E+1] (exclusive scan, offset[E] = A),
 *   perm [A] (perm[p] = assignment at bucket position p),
 *   inv_perm [A] (inv_perm[i] = bucket position of assignment i)  -- outputs
 * An index outside [0,E) is not detected at enqueue time; such an assignment
 * is dropped from every bucket and its inv_perm entry is set to -1.
 * Precondition for what consumes the buckets: the k indices of a token are
 * distinct (moe_route guarantees it), so that no bucket holds more than T rows. */
moe_status moe_permute(const moe_shape* shape, const int32_t* topk_idx,
                       int32_t* count, int32_t* offset, int32_t* perm,
                       int32_t* inv_perm, void* stream);

/* Re-layout of one bf16 matrix [N,K] (row-major, device) into MOE_TILED form
 * (device, a different buffer of the same size).  N a multiple of 16, K of 32.
 * Not a hot call. */
moe_status moe_pack_weights(const void* src, void* dst, int32_t N, int32_t K, void* stream);

/* ---- a4: grouped SiLU-gated expert FFN over the active experts -----------
 * Section 4.4's three matrices per expert.  For every expert e < E whose bit is
 * set in the mask and whose bucket is not empty, and for every bucket position
 * p in [offset[e], offset[e+1]) with token t = perm[p] / k:
 *     h = silu(Wg_e . x_t) * (Wu_e . x_t),   Y[p,:] = Wd_e . h
 * and for every shared expert s < S whose bit (E+s) is set, for every token t:
 *     Y[A + s*T + t, :] = FFN_{E+s}(x_t).
 * Experts with an empty bucket or a cleared bit read no weight bytes and leave
 * their rows of Y untouched.
 * Precondition: no bucket holds more than T rows (true whenever a token's k
 * experts are distinct, as moe_route produces them).  The kernels size their
 * grids by T; rows of a bucket beyond its first T are not computed and their
 * rows of Y stay untouched.  This cannot be checked at enqueue time.
 *   X [T,H] storage dtype; perm [A], offset [E+1] as produced by moe_permute
 *   host_experts: HOST array [E+S] of device pointers (copied at enqueue time;
 *                 entries of experts excluded by the mask may be NULL)
 *   host_expert_mask: HOST array of ceil((E+S)/64) words, bit e of word e/64;
 *                 NULL = all experts
 *   Y [A + S*T, H] float32 (output)
 *   workspace: device scratch of moe_workspace_bytes(shape) bytes (holds h;
 *              bf16 storage rounds h to bfloat16 once, nearest even)
 */
moe_status moe_grouped_ffn(const moe_shape* shape, const void* X,
                           const int32_t* perm, const int32_t* offset,
                           const moe_expert_ptrs* host_experts,
                           const uint64_t* host_expert_mask, float* Y,
                           void* workspace, void* stream);

/* ---- a5: weighted combine back to token order ----------------------------
 * Section 2.1: x' = sum_j w_j * Expert_j(a).
 *   out[t,:] = sum_{j<k} topk_w[t,j] * Y[inv_perm[t*k+j], :]
 *            + sum_{s<S} Y[A + s*T + t, :]  (+ residual[t,:])
 * summed in float32 in exactly that order, rounded once to the storage dtype.
 *   residual [T,H] storage dtype or NULL;  out [T,H] storage dtype. */
moe_status moe_combine(const moe_shape* shape, const float* Y,
                       const float* topk_w, const int32_t* inv_perm,
                       const void* residual, void* out, void* stream);

/* ---- a6: context for expert streaming ------------------------------------
 * Section 4.4: fixed device slots registered once, so that moving an expert is
 * an overwrite of an existing buffer and nothing is allocated per transfer.
 * moe_create allocates `n_ondemand_slots` (>= 2: one computing, one loading)
 * plus 2 * `n_prefetch_slots_per_group` slots (group "current layer" and group
 * "next layer", rotated after every layer), each big enough for one expert of
 * `max_shape` (3*H*F elements), one side stream at default priority, events,
 * and a small pinned host buffer for the per-expert counts.  Both slot counts
 * may be 0 if every expert will always be resident.  Not a hot call. */
moe_status moe_create(const moe_shape* max_shape, int32_t n_ondemand_slots,
                      int32_t n_prefetch_slots_per_group, moe_ctx** out_ctx);

/* Waits for the context's streams, frees slots, streams and events. */
moe_status moe_destroy(moe_ctx* ctx);

/* One layer's weights.  host arrays are indexed by expert, routed experts
 * first, then shared experts. */
typedef struct {
  const void* Wr;                      /* [E,H] device                        */
  const float* bias;                   /* [E] device or NULL                  */
  const moe_expert_ptrs* host_dev;     /* HOST array [E+S]: device-resident
                                          copies (entries of non-resident
                                          experts are ignored)                */
  const moe_expert_ptrs* host_pinned;  /* HOST array [E+S]: pinned host copies
                                          (needed for non-resident experts;
                                          may be NULL if all are resident)    */
  uint64_t layer_id;                   /* names the layer in slot tags        */
} moe_layer_desc;

/* Filled on the host before moe_layer_forward returns. */
typedef struct {
  int32_t n_active;        /* routed experts with a non-empty bucket; -1 if the
                              call did not need to read the counts back       */
  int32_t n_resident;      /* active and resident                             */
  int32_t n_hit;           /* active, non-resident, found in a prefetch slot  */
  int32_t n_miss;          /* active, non-resident, loaded on demand          */
  int32_t n_wasted;        /* prefetched for this layer but not active        */
  int32_t n_prefetch_issued; /* copies started for the next layer             */
  int64_t bytes_on_demand; /* host-to-device bytes queued on demand           */
  int64_t bytes_prefetch;  /* host-to-device bytes queued as prefetch         */
} moe_layer_stats;

/* ---- the whole block ------------------------------------------------------
 * route -> permute -> grouped FFN -> combine for one layer, with experts taken
 * from wherever they live:
 *   resident (bit set in host_resident_mask): computed first, from host_dev;
 *   not resident, but prefetched for this layer_id into the current prefetch
 *     group: a hit, computed from the slot once its copy has landed;
 *   not resident, no slot: a miss, copied on demand through the on-demand
 *     double buffer, queued AHEAD of any prefetch issued by this call;
 *   empty bucket: skipped, nothing read, nothing copied.
 * After the on-demand copies, copies of `host_prefetch_next_mask`'s experts of
 * `next_layer` are queued into the next-layer prefetch group; after the layer
 * the two groups swap roles.  Shared experts must be resident.
 * If a routed expert is neither resident nor in a prefetch slot for this
 * layer, or if stats are requested, the call waits (on the host) for the
 * router's counts before it can queue copies; with every expert resident or
 * prefetched and stats == NULL it never blocks.
 *   out = block output (+ residual if given), [T,H] storage dtype.
 * Rounding points between the router and `out` (bf16 storage): h is rounded to
 * bf16 once; the rows of Y stay float32 up to the combine -- except at the
 * shapes for which moe_layer_y_dtype() answers MOE_BF16 (prefill sizes: about
 * a hundred rows per expert and more), where each expert's output row is
 * rounded to bf16 before the weighted sum, as a model that runs its experts as
 * separate bf16 modules does; the sum itself is float32 and rounded once.
 *   host_resident_mask / host_prefetch_next_mask: HOST words, ceil(E/64) each;
 *     NULL resident mask = all resident; NULL prefetch mask = none.
 *   next_layer may be NULL.  stats may be NULL. */
moe_status moe_layer_forward(moe_ctx* ctx, const moe_shape* shape,
                             const moe_layer_desc* layer,
                             const uint64_t* host_resident_mask,
                             const moe_layer_desc* next_layer,
                             const uint64_t* host_prefetch_next_mask,
                             const void* X, const void* residual, void* out,
                             void* workspace, void* stream,
                             moe_layer_stats* stats);

/* The prefetch step of moe_layer_forward as a call of its own, for a scheduler
 * that decides the prefetch set while the current layer is already queued
 * (Section 4.3: the decision for layer l+1 uses what layer l's gate has just
 * activated; Section 4.4: prefetches run on the side stream behind the
 * on-demand loads).  Call it after the moe_layer_forward of layer l (given no
 * prefetch mask) and before that of layer l+1: it queues the copies of
 * `next_layer`'s experts named in host_prefetch_mask (HOST words, ceil(E/64);
 * ascending expert order, as many as a prefetch group has slots) into the
 * group the next moe_layer_forward call reads, behind every copy queued so
 * far, and drops what that group held.  Never blocks on the GPU.
 *   *n_issued (may be NULL) receives the number of copies queued.
 * Errors: NULL argument, expert without a pinned copy, expert larger than the
 * context's slots. */
moe_status moe_prefetch(moe_ctx* ctx, const moe_shape* shape, const moe_layer_desc* next_layer,
                        const uint64_t* host_prefetch_mask, void* stream, int32_t* n_issued);

/* The per-expert token counts of the layer the last moe_layer_forward call
 * ran (the pending tokens per expert of Section 4.3.2, Premise 1), for a
 * scheduler on the host.  Needs MOE_OPT_EXPORT_COUNTS: every layer call then
 * queues a copy of its E counts to pinned host memory right behind the
 * bucketing kernel and goes on without waiting; this call waits for that copy
 * (the layer's routing and bucketing, not its FFN) and hands the counts over.
 *   host_count [E] int32, E = the shape's routed experts.
 * Errors: option not set / no layer run yet, E differs from the last layer's. */
moe_status moe_layer_counts(moe_ctx* ctx, int32_t* host_count, int32_t E);

/* ---- the block, for callers that cannot allocate ---------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that
 * forbid hipMalloc: the same block as moe_layer_forward for a layer whose
 * experts are ALL resident (every entry of layer->host_dev non-NULL), with no
 * workspace argument and no context.  The intermediate buffers (top-k lists,
 * bucket offsets and permutations, router logits, h, Y) live in a fixed device
 * array of MOE_STATIC_WORKSPACE_BYTES inside the library; each GPU the library
 * runs on holds its own copy of it until the process ends.  The call allocates
 * nothing: no hipMalloc / hipFree, no events, no streams.  Its output is bit
 * for bit that of moe_layer_forward on the same inputs.
 *   - MOE_ERR_WORKSPACE if moe_workspace_bytes(shape) - 256 exceeds the array
 *     (e.g. the Mixtral-shaped layer fits up to 128 tokens, not 256);
 *   - every call on a GPU shares that GPU's array: calls that overlap in time
 *     on one GPU (two streams, two threads) race; serialise them.  Nothing in
 *     the array has to start at zero and nothing is kept between calls.
 *   X, residual (nullable), out: as moe_layer_forward. */
#define MOE_STATIC_WORKSPACE_BYTES (16u << 20)
size_t moe_static_workspace_bytes(void);
moe_status moe_layer_forward_static(const moe_shape* shape, const moe_layer_desc* layer,
                                    const void* X, const void* residual, void* out,
                                    void* stream);

/* Stack glue (outside the block itself): weightless RMS normalisation of the
 * residual stream, out[t,:] = X[t,:] / sqrt(mean_h X[t,h]^2 + eps), float32
 * arithmetic, one rounding to the storage dtype.  A stack of MoE blocks is
 * x_{l+1} = x_l + Block_l(rmsnorm(x_l)): call this, then moe_layer_forward
 * with `residual` = x_l.  X, out [T,H] storage dtype (may not alias). */
moe_status moe_rmsnorm(const moe_shape* shape, const void* X, void* out, float eps, void* stream);

/* Host-side totals of the context's side stream since creation (or the last
 * reset): bytes copied and the summed duration of the copies as measured by
 * event pairs around each one.  Synchronises the side stream. */
typedef struct {
  int64_t bytes;
  int64_t n_copies;
  double copy_ms;
} moe_stream_totals;
moe_status moe_stream_totals_get(moe_ctx* ctx, moe_stream_totals* out, int32_t reset);

/* Context options.
 * MOE_OPT_SYNC_COPIES (default 0): with a non-zero value every expert copy
 *   waits for the compute stream to drain first and is waited for before
 *   anything else is queued, i.e. no copy overlaps any compute (the
 *   "synchronous loading" Section 4.4 compares against).  A control for
 *   measurements; results are unchanged.
 * MOE_OPT_COPY_SPLIT (default 1): 1 = an expert whose three matrices are
 *   contiguous in pinned host memory (Wu = Wg + H*F elements, Wd = Wu + H*F)
 *   moves as one copy; 3 = one copy per matrix in need order (gate, up, down)
 *   with the first FFN phase gated on gate+up only (Section 4.4's sub-tensor
 *   granularity).  Non-contiguous experts always move as three copies.
 * MOE_OPT_EXPORT_COUNTS (default 0): non-zero = every moe_layer_forward call
 *   also copies its per-expert token counts to the host (see moe_layer_counts). */
typedef enum { MOE_OPT_SYNC_COPIES = 0, MOE_OPT_COPY_SPLIT = 1, MOE_OPT_EXPORT_COUNTS = 2 } moe_option;
moe_status moe_set_option(moe_ctx* ctx, int32_t option, int64_t value);

/* Optional per-phase timing of layers whose experts are all resident, for
 * measurement harnesses; off by default.
 *   mode 1: moe_layer_forward records an event on `stream` before the router
 *           and after each of the five kernels (route, permute, gate/up, down,
 *           combine): six markers per layer;
 *   mode 2: only the two markers around the gate/up kernel (the dominant one),
 *           which perturbs the layer's own timing less (about 5 us per layer);
 *   mode 3: as mode 2, on every fourth call only (the first after the mode was
 *           set, then every fourth): a sample of the launches of a timed
 *           region at a quarter of the cost;
 *   mode 0: off.
 * moe_phase_times_get waits for the recorded layers and returns the summed
 * durations: the five phases over `n_layers` mode-1 layers, and
 * `gate_up_only_ms` over `gate_up_only_layers` layers marked in mode 2 or 3. */
typedef struct {
  double route_ms, permute_ms, gate_up_ms, down_ms, combine_ms;
  int64_t n_layers;
  double gate_up_only_ms;
  int64_t gate_up_only_layers;
} moe_phase_times;
moe_status moe_phase_timing(moe_ctx* ctx, int32_t mode);
moe_status moe_phase_times_get(moe_ctx* ctx, moe_phase_times* out, int32_t reset);

/* Measurement aids (not part of the method): a plain streaming copy
 * dst[0:bytes] = src[0:bytes] and a plain streaming read of src[0:bytes]
 * (sink4: 4 bytes of device scratch), 16 bytes per lane; `bytes` a multiple of
 * 16.  They give the box's achievable HBM rate and a dispatch of known size
 * for scaling hardware byte counters. */
moe_status moe_probe_copy(void* dst, const void* src, size_t bytes, void* stream);
moe_status moe_probe_read(const void* src, size_t bytes, void* sink4, void* stream);
/* The same bytes read with non-temporal loads (the hint the FFN kernels put on
 * weight tiles that are read once), eight 1 KiB loads in flight per wavefront
 * over 8 KiB in a row. */
moe_status moe_probe_read_nt(const void* src, size_t bytes, void* sink4, void* stream);
/* The stage loop of the tiled FFN kernels with nothing multiplied: 256
 * workgroups of eight waves, each streaming `stages` x 16 KiB of its own out of
 * `weights` (device, at least 256 x stages x 16 KiB, non-temporal loads) while
 * it fetches token_fetches x 8 KiB per stage (0..4; 8 rows x 128 B per
 * instruction) out of `tokens` (device, at least 2 MiB: 256 rows of 8 KiB, which
 * stay in L2), direct-to-LDS into a ring with two stages in flight.  Timed by
 * the caller, it shows how far bytes that hit in L2 slow an HBM-bound weight
 * stream down.  Nothing is written to global memory.  MOE_ERR_INVALID_ARG for
 * buffers that are too small or arguments out of range. */
moe_status moe_probe_stage(const void* weights, size_t weight_bytes, const void* tokens,
                           size_t token_bytes, int32_t token_fetches, int32_t stages, void* stream);

/* Which kernel the grouped FFN launches for a shape (measurement aid for
 * reports): phase 0 = gate/up, 1 = down.  The choice depends on the shape
 * alone; n_groups (experts listed in a call) is accepted and ignored, so a
 * call over a subset of experts runs the same kernels, bit for bit, as a call
 * over all of them.  Returns a static string, "" for an invalid request. */
const char* moe_ffn_kernel_name(const moe_shape* shape, int32_t phase, int32_t n_groups);

/* Element type of the rows of Y that moe_layer_forward (and
 * moe_layer_forward_static) keeps in the workspace between the down projection
 * and the combine for `shape`: MOE_F32, or MOE_BF16 where the down projection
 * runs its prefill form (there Y is the largest tensor the block writes and
 * reads back, and half its bytes are worth more than its last mantissa bits: the
 * block's output stays within the bf16 tolerance either way).  Depends on the
 * shape alone.  moe_grouped_ffn and moe_combine always exchange float32 rows.
 * Returns -1 for an invalid shape. */
int32_t moe_layer_y_dtype(const moe_shape* shape);

/* Views into a workspace after moe_layer_forward (device pointers into
 * `workspace`; for tests and harnesses).  Any output pointer may be NULL.
 * *Y points at [T*k + S*T, H] rows of the type moe_layer_y_dtype() names. */
moe_status moe_workspace_views(const moe_shape* shape, void* workspace,
                               int32_t** topk_idx, float** topk_w,
                               int32_t** count, int32_t** offset,
                               int32_t** perm, int32_t** inv_perm, void** Y);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HOTPATH_H */
