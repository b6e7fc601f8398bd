/*
 * moe_sched.h -- C ABI of the scheduling side of the MoE hot path: what decides
 * WHICH experts' bytes move, never what the block computes.
 *
 *  - the hot-expert table (Section 4.1): a counter of tokens processed per
 *    expert, and the choice of resident experts under a memory budget;
 *  - a gate-based expert predictor (the strategy of Section 3.2 / Figure 6):
 *    the next layer's router applied to the current layer's input;
 *  - PreSched (Section 4.3): the cross-layer queue (Q1, Eq. 3), the local
 *    recheck (Eq. 4), the prefetch count (Q2, Eq. 5), the critical-prefetch
 *    rule (Q3, Eq. 6) and the no-benefit exit (Q4), with the CPU cost model of
 *    Eq. 2.
 *
 * Conventions are those of moe_hotpath.h: device pointers unless the name
 * starts with `host_`; every call returns a moe_status; moe_last_error() has
 * the reason.  The two host-only calls (moe_hot_table, moe_presched) touch no
 * GPU and may be called without one.
 */
#ifndef MOE_SCHED_H
#define MOE_SCHED_H

#include "moe_hotpath.h"

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_SCHED_MAX_EXPERTS 128

/* The Counter of Section 4.1: total[e] += count[e] for e < shape->E, on the
 * device.  `count` is the per-expert token count moe_permute / moe_layer_forward
 * leave in the workspace; `total` [E] int64 is owned and zeroed by the caller. */
moe_status moe_counter_add(const moe_shape* shape, const int32_t* count, int64_t* total,
                           void* stream);

/* Hot-expert table (Section 4.1): rank all L*E experts by tokens processed and
 * mark the hottest resident, in descending order, until `budget_experts`
 * (equally sized) experts are placed.  Equal counts: lower layer, then lower
 * expert index first.  host_tokens [L*E] row-major by layer;
 * host_resident [L*E] receives 1 (resident) or 0.  budget <= 0 marks none,
 * budget >= L*E marks all.  Errors: NULL pointer, L < 1, E < 1. */
moe_status moe_hot_table(const int64_t* host_tokens, int32_t L, int32_t E,
                         int64_t budget_experts, uint8_t* host_resident);

/* Gate-based prediction of the next layer's pending tokens per expert: routes
 * X [T,H] (the CURRENT layer's input) with the NEXT layer's router
 * (Wr_next [E,H], bias_next [E] or NULL) exactly as moe_route does, and writes
 * how many (token, slot) assignments each expert receives to pred_count [E].
 * Uses the routing part of `workspace` (moe_workspace_bytes(shape)) as scratch:
 * call it before moe_layer_forward on the same stream, or with a workspace of
 * its own. */
moe_status moe_predict_counts(const moe_shape* shape, const void* X, const void* Wr_next,
                              const float* bias_next, int32_t* pred_count, void* workspace,
                              void* stream);

/* The pending experts of a layer for a scheduling decision (Premise 1 of
 * Section 4.3.2: experts that are activated, or predicted, and are neither on
 * the GPU nor being loaded): every e < E with host_count[e] > 0 whose bit is
 * clear in host_resident_mask and in host_in_flight_mask.  Host only.
 *   host_count [E] tokens per expert (activated or predicted)
 *   host_resident_mask, host_in_flight_mask: ceil(E/64) words, bit e of word
 *     e/64; either may be NULL (= no expert resident / none in flight)
 *   host_pending [E] receives the entries by ascending expert id,
 *   *n_pending their number.
 * Errors: NULL count / output, E outside [1, 128], a negative count. */
typedef struct { int32_t expert; int32_t tokens; } moe_pending;
moe_status moe_pending_experts(const int32_t* host_count, int32_t E,
                               const uint64_t* host_resident_mask,
                               const uint64_t* host_in_flight_mask,
                               moe_pending* host_pending, int32_t* n_pending);

/* Fixed-count prefetch policy (the one Section 5.3's ablation falls back to
 * without PreSched: a fixed number of experts per layer): the n_prefetch
 * pending experts with the most tokens, equal counts by ascending expert id,
 * hottest first.  Host only.
 *   host_chosen [min(n_prefetch, n_pending)] expert ids in issue order,
 *   *n_chosen their number.  n_prefetch <= 0 chooses none.
 * Errors: NULL pointer with a positive length, n_pending outside [0, 128]. */
moe_status moe_prefetch_hottest(const moe_pending* host_pending, int32_t n_pending,
                                int32_t n_prefetch, int32_t* host_chosen, int32_t* n_chosen);

/* Cost inputs of PreSched (Section 4.3.2, "Constraints"); any time unit, used
 * consistently.  t_c(m) = beta*m + C is Eq. 2. */
typedef struct {
  double t_io;          /* load time of one expert over the host link (> 0) */
  double t_g;           /* GPU compute time of one expert (token-invariant)  */
  double t_attn;        /* attention time of a layer                         */
  double beta;          /* CPU cost per token                                */
  double C;             /* CPU start-up cost per expert                      */
  double alpha;         /* delay of the first on-demand load behind a prefetch in flight */
  double r_hit;         /* hit rate of the critical prefetch in [0,1]; miss rate = 1 - r_hit */
  int32_t cpu_executor; /* 1: experts left on the host are computed there (the paper's setting).
                           0: GPU-only: every pending expert of the current layer is
                              loaded, the queue holds all of E_all and i' = 0 */
} moe_presched_costs;

/* moe_pending (above): one expert that is activated (current layer) or predicted
 * (next layer) and is neither on the GPU nor being loaded (Premise 1). */

typedef struct {
  int32_t n_cur, n_next;                      /* n + 1 and n' of the paper              */
  int32_t cur_sorted[MOE_SCHED_MAX_EXPERTS];  /* E_cur: expert ids, ascending tokens    */
  int32_t next_sorted[MOE_SCHED_MAX_EXPERTS]; /* E_next                                 */
  int32_t n_all;                              /* n + n' + 1                             */
  int32_t all_layer[2 * MOE_SCHED_MAX_EXPERTS];   /* E_all: 0 = current, 1 = next layer */
  int32_t all_expert[2 * MOE_SCHED_MAX_EXPERTS];
  int32_t all_in_queue[2 * MOE_SCHED_MAX_EXPERTS]; /* 1 when E_all[i] is in GPU_Q       */
  int32_t i_prime;                            /* E_cur[i'..n] load on demand; n+1 = none */
  int32_t n_ondemand;
  int32_t ondemand[MOE_SCHED_MAX_EXPERTS];    /* expert ids in load order               */
  double T_gap;                               /* link window left by the current layer  */
  double f;                                   /* Eq. 5                                  */
  int32_t f_abs;                              /* f rounded half up, clamped to [0, n']  */
  double xi;                                  /* Eq. 6, benefit of the critical prefetch */
  int32_t n_prefetch;
  int32_t prefetch[MOE_SCHED_MAX_EXPERTS];    /* expert ids in issue order, hottest first */
} moe_presched_plan;

/* One PreSched decision for a layer (host only).  Lists are sorted by
 * ascending pending tokens, equal counts by ascending expert id; in the merged
 * list a next-layer expert sorts below a current-layer expert with the same
 * count.  GPU_Q: E_all[i] with  alpha + (n+n'-i+1) t_io + t_g  <
 * t_c(E_all[0..i]) + t_attn.  i': smallest index of E_cur that is in GPU_Q and
 * has  alpha + (n-i'+1) t_io + t_g  <  t_c(E_cur[0..i'-1]);  none: i' = n+1.
 * T_gap = t_c(E_cur[0..i'-1]) - alpha - (n-i'+1) t_io;  f = (T_gap + t_attn)/t_io.
 * When GPU_Q holds no next-layer expert nothing is prefetched; otherwise |f|
 * experts when  r_hit (f-|f|+1) > (1-r_hit)(|f|-f),  else |f|-1, the hottest
 * of E_next, hottest first.
 * Errors: NULL pointer, n_cur or n_next outside [0, 128], t_io <= 0, a
 * negative token count, r_hit outside [0,1]. */
moe_status moe_presched(const moe_presched_costs* host_costs, const moe_pending* host_cur,
                        int32_t n_cur, const moe_pending* host_next, int32_t n_next,
                        moe_presched_plan* host_plan);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SCHED_H */
