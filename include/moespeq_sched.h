/*
 * moespeq_sched.h - host-side control plane of the MoE draft/verify path (C ABI, no GPU work):
 * the Speculative Governor (paper section 3.2) and the Expert Scheduler (section 3.3).
 *
 * Every pointer in this header is a HOST pointer.  Functions return MOE_OK (0) or a negative
 * MOE_ERR_* status from moespeq.h; nothing here touches a device or a stream, allocates only in
 * the *_create calls, and is not thread-safe per object (one caller per object at a time).
 */
#ifndef MOESPEQ_SCHED_H
#define MOESPEQ_SCHED_H

#include <stddef.h>
#include <stdint.h>
#include "moespeq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- Speculative Governor (section 3.2) --------------------------------------------------- */

typedef struct moe_governor moe_governor;

/*
 * Profiled constants of the Amortization Roofline Model (section 3.2.2, "Latency and I/O
 * Modeling").  Times in seconds, sizes in bytes.
 */
typedef struct {
    double t_draft_base, t_draft_token; /* T_draft(k) = base + k * token                              */
    double t_pcie_init;                 /* T_pcie,init: latency of the first mandatory expert fetch   */
    double t_pcie_overhead;             /* fixed part of T_pcie,new (charged only when n_new > 0)     */
    double b_pcie;                      /* effective host-to-device bandwidth, bytes/s, > 0           */
    double s_expert;                    /* bytes of one expert, > 0                                   */
    int32_t n_verify;                   /* >= 1 profiled points of T_verify                           */
    const int32_t *verify_tokens;       /* [n_verify] strictly ascending token counts (k + 1)         */
    const double *verify_seconds;       /* [n_verify] T_verify at those counts                        */
    double ema_alpha;                   /* weight of a new acceptance observation, in (0, 1]          */
    double p_init;                      /* acceptance probabilities before any observation, in [0, 1] */
    int32_t k_min, k_max;               /* 1 <= k_min <= k_max <= MOE_GOVERNOR_MAX_K                  */
} moe_governor_config;

#define MOE_GOVERNOR_MAX_K 64

/* Copies the configuration (including the two arrays).  MOE_ERR_INVALID_ARG on any violated
 * bound above. */
int moe_governor_create(moe_governor **out, const moe_governor_config *cfg);
int moe_governor_destroy(moe_governor *g);

/*
 * One finished cycle: `drafted` tokens were proposed, the first `accepted` of them were accepted
 * (0 <= accepted <= drafted <= k_max).  p_i is the probability that token i is accepted given that
 * tokens 1..i-1 were (section 3.2.2): positions 1..accepted observe 1, position accepted+1 (if it
 * was drafted) observes 0, later positions were not reached and keep their value.  Each observed
 * p_i becomes (1 - alpha) * p_i + alpha * observation (exponential moving average).
 */
int moe_governor_observe(moe_governor *g, int32_t drafted, int32_t accepted);
/* p[0..k_max-1] = p_1..p_{k_max}. */
int moe_governor_probabilities(const moe_governor *g, double *p);

/* k_accept(k) = sum_{i=1..k} prod_{j=1..i} p_j  (expected accepted tokens, Eq. 2's numerator). */
int moe_governor_k_accept(const moe_governor *g, int32_t k, double *k_accept);

/*
 * Eq. 3: T_cycle(k) = max(T_draft(k), T_pcie,init) + T_pcie,new(k) + T_verify(k + 1) with
 * T_pcie,new = 0 if n_new == 0 else t_pcie_overhead + n_new * s_expert / b_pcie, and T_verify
 * interpolated linearly between the profiled points (extended with the slope of the first / last
 * segment outside them; constant if there is one point).  n_new = |E_new(k)|, the experts of the
 * draft window that are not in the cache (moe_expert_union's n_missing summed over the layers).
 */
int moe_governor_cycle_time(const moe_governor *g, int32_t k, int32_t n_new, double *t_cycle);

/*
 * The operating point of draft length k: theta = k_accept / T_cycle (Eq. 2, accepted tokens per
 * second) and the amortization intensity (Eq. 1, S_token = 1) = k_accept / (n_new * s_expert),
 * +infinity when n_new == 0.  Either output may be NULL.
 */
int moe_governor_evaluate(const moe_governor *g, int32_t k, int32_t n_new, double *theta, double *intensity);

/*
 * Eq. 4 / 5: k* = argmax over k in [k_min, min(k_max, k_slo)] of theta(k) (the smallest such k on
 * ties; the paper's last equation names the objective differently, it is read as the same theta).
 * n_new_by_k[k] for k = 0..k_max is |E_new(k)| (entry 0 is ignored).  k_slo <= 0 means no
 * service-level bound.  MOE_ERR_INVALID_ARG if the range is empty.
 */
int moe_governor_choose_k(const moe_governor *g, const int32_t *n_new_by_k, int32_t k_slo,
                          int32_t *k_star, double *theta_star);

/* ---- Expert Lookahead Buffer (section 3.3.1) ------------------------------------------------ */

typedef struct moe_elb moe_elb;

/*
 * The ELB of one speculative window: for each draft token (step) and MoE layer the top_k
 * (expert id, confidence) pairs the draft pass emitted (moe_draft_layer_int4's ids_out / conf_out,
 * copied to the host by the caller, one copy per step or per window).
 * 1 <= n_layers, 1 <= k_max <= MOE_GOVERNOR_MAX_K, 1 <= top_k <= MOE_MAX_TOPK.
 */
int moe_elb_create(moe_elb **out, int32_t n_layers, int32_t k_max, int32_t top_k);
int moe_elb_destroy(moe_elb *elb);
/* Starts a new window: no step is filled. */
int moe_elb_reset(moe_elb *elb);
/* Entries of draft token `step` for all layers: ids / conf are [n_layers, top_k]; conf may be NULL
 * (recorded as 1).  Steps arrive in order: step must equal the number of steps filled so far. */
int moe_elb_put_step(moe_elb *elb, int32_t step, const int32_t *ids, const float *conf);
int moe_elb_steps(const moe_elb *elb, int32_t *n_steps);
/* Reads one entry back: ids [top_k], conf [top_k] (conf may be NULL). */
int moe_elb_entry(const moe_elb *elb, int32_t step, int32_t layer, int32_t *ids, float *conf);

/* ---- Expert cache: slot tables with lookahead-aware eviction (section 3.3.2) ---------------- */

typedef struct moe_cache moe_cache;

/* One slot pool of n_slots slots per layer, all empty.  1 <= n_experts <= MOE_MAX_EXPERTS,
 * 1 <= n_slots <= n_experts. */
int moe_cache_create(moe_cache **out, int32_t n_layers, int32_t n_experts, int32_t n_slots);
int moe_cache_destroy(moe_cache *c);
/* Initial residency: `expert` sits in `slot` of `layer` (the slot must be empty, the expert absent). */
int moe_cache_place(moe_cache *c, int32_t layer, int32_t expert, int32_t slot);
/* slot_of_expert[e] for e < n_experts, -1 = absent: the table moe_verify_layer_bf16 takes (the caller
 * copies it to the device). */
int moe_cache_slot_table(const moe_cache *c, int32_t layer, int32_t *slot_of_expert);
/*
 * The verify call of `layer` needs these experts (n ids, duplicates allowed).  Counts every distinct
 * one as a hit (resident) or a miss, adds them to the running totals and makes them the most
 * recently used of the layer.  n_hit / n_miss may be NULL.
 */
int moe_cache_use(moe_cache *c, int32_t layer, const int32_t *ids, int32_t n, int32_t *n_hit, int32_t *n_miss);
/* Totals over all moe_cache_use calls: the per-step cache coverage of the paper's Table 3 is
 * hits / (hits + misses). */
int moe_cache_stats(const moe_cache *c, int64_t *hits, int64_t *misses);
/* Ends the speculative window: no expert is protected from eviction any more. */
int moe_cache_end_window(moe_cache *c);

/* One expert to copy: fill `slot` of `layer` with `expert`; `evicted` is the expert that was there
 * (-1: the slot was empty).  The cache already counts the expert as resident. */
typedef struct { int32_t layer, expert, slot, evicted; } moe_fetch;

#define MOE_PHASE_PRIME    1   /* Phase I: serve from the cache, fetch nothing                 */
#define MOE_PHASE_GUIDED   2   /* Phase II: a budgeted subset of the predicted experts         */
#define MOE_PHASE_SATURATE 3   /* Phase III: every predicted expert that is still missing      */

/*
 * The three-phase prefetch of section 3.3.2 over the steps the ELB holds so far.  Every expert the
 * ELB names becomes protected: it is not evicted before moe_cache_end_window.
 *   PRIME     nothing is fetched (n_out = 0): resident predicted experts are only protected.
 *   GUIDED    missing predicted experts in the order (layer, confidence descending, expert id), at
 *             most max_fetch of them and only those with confidence >= min_conf (an expert's
 *             confidence is the largest one any ELB entry gives it).
 *   SATURATE  all missing predicted experts in the order (layer, expert id); max_fetch and min_conf
 *             are ignored.
 * Slot choice: an empty slot of the layer if there is one (lowest first), else the least recently
 * used unprotected expert of the layer; if every slot holds a protected expert the fetch is skipped
 * (the verify call will report the expert missing).  The paper does not specify the eviction rule
 * beyond "lookahead-aware": this is Belady's rule on the lookahead the ELB gives (an expert the
 * window needs is needed sooner than one it does not name), with recency among the rest.
 * out: [max_out]; MOE_ERR_WORKSPACE if more than max_out fetches are due (none is applied then).
 */
int moe_sched_plan(moe_cache *c, const moe_elb *elb, int32_t phase, int32_t max_fetch, float min_conf,
                   moe_fetch *out, int32_t max_out, int32_t *n_out);
/*
 * On-demand path: the verify call of `layer` reported `missing` (n distinct absent experts).  Each
 * gets a slot: an empty one, else the least recently used expert of the layer that is not itself in
 * `missing` (protected or not: what the first pass needed has been used).  out: [n].
 * MOE_ERR_WORKSPACE if n exceeds the layer's slots.
 */
int moe_sched_on_demand(moe_cache *c, int32_t layer, const int32_t *missing, int32_t n, moe_fetch *out);

#ifdef __cplusplus
}
#endif
#endif /* MOESPEQ_SCHED_H */
