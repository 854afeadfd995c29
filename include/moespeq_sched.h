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

#ifdef __cplusplus
}
#endif
#endif /* MOESPEQ_SCHED_H */
