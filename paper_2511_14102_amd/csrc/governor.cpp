// Speculative Governor (paper section 3.2): the Amortization Roofline Model as plain host
// arithmetic behind the C ABI of include/moespeq_sched.h.
#include <cmath>
#include <limits>
#include <new>
#include <vector>
#include "../../include/moespeq_sched.h"

struct moe_governor {
    moe_governor_config cfg;
    std::vector<int32_t> vtok;
    std::vector<double> vsec;
    std::vector<double> p;          // p[i-1] = p_i
};

namespace {

bool finite_nonneg(double v) { return std::isfinite(v) && v >= 0.0; }

double verify_time(const moe_governor *g, double tokens)
{
    const size_t n = g->vtok.size();
    if (n == 1) return g->vsec[0];
    size_t hi = 1;                                   // segment [hi-1, hi] that holds (or is nearest to) tokens
    while (hi + 1 < n && tokens > (double)g->vtok[hi]) ++hi;
    const double x0 = g->vtok[hi - 1], x1 = g->vtok[hi];
    return g->vsec[hi - 1] + (g->vsec[hi] - g->vsec[hi - 1]) * (tokens - x0) / (x1 - x0);
}

double k_accept(const moe_governor *g, int k)
{
    double sum = 0.0, prod = 1.0;
    for (int i = 0; i < k; ++i) { prod *= g->p[i]; sum += prod; }
    return sum;
}

double cycle_time(const moe_governor *g, int k, int n_new)
{
    const moe_governor_config &c = g->cfg;
    const double t_draft = c.t_draft_base + k * c.t_draft_token;
    const double t_new = n_new == 0 ? 0.0 : c.t_pcie_overhead + n_new * c.s_expert / c.b_pcie;
    return std::fmax(t_draft, c.t_pcie_init) + t_new + verify_time(g, k + 1);
}

}  // namespace

extern "C" {

int moe_governor_create(moe_governor **out, const moe_governor_config *cfg)
{
    if (!out || !cfg) return MOE_ERR_INVALID_ARG;
    const moe_governor_config &c = *cfg;
    if (!finite_nonneg(c.t_draft_base) || !finite_nonneg(c.t_draft_token) || !finite_nonneg(c.t_pcie_init) ||
        !finite_nonneg(c.t_pcie_overhead) || !(std::isfinite(c.b_pcie) && c.b_pcie > 0.0) ||
        !(std::isfinite(c.s_expert) && c.s_expert > 0.0))
        return MOE_ERR_INVALID_ARG;
    if (c.n_verify < 1 || !c.verify_tokens || !c.verify_seconds) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < c.n_verify; ++i) {
        if (!finite_nonneg(c.verify_seconds[i]) || c.verify_tokens[i] < 1) return MOE_ERR_INVALID_ARG;
        if (i && c.verify_tokens[i] <= c.verify_tokens[i - 1]) return MOE_ERR_INVALID_ARG;
    }
    if (!(c.ema_alpha > 0.0 && c.ema_alpha <= 1.0) || !(c.p_init >= 0.0 && c.p_init <= 1.0))
        return MOE_ERR_INVALID_ARG;
    if (c.k_min < 1 || c.k_min > c.k_max || c.k_max > MOE_GOVERNOR_MAX_K) return MOE_ERR_INVALID_ARG;
    moe_governor *g = new (std::nothrow) moe_governor;
    if (!g) return MOE_ERR_HIP;
    g->cfg = c;
    g->vtok.assign(c.verify_tokens, c.verify_tokens + c.n_verify);
    g->vsec.assign(c.verify_seconds, c.verify_seconds + c.n_verify);
    g->cfg.verify_tokens = nullptr;
    g->cfg.verify_seconds = nullptr;
    g->p.assign(c.k_max, c.p_init);
    *out = g;
    return MOE_OK;
}

int moe_governor_destroy(moe_governor *g)
{
    delete g;
    return MOE_OK;
}

int moe_governor_observe(moe_governor *g, int32_t drafted, int32_t accepted)
{
    if (!g || accepted < 0 || accepted > drafted || drafted > g->cfg.k_max) return MOE_ERR_INVALID_ARG;
    const double a = g->cfg.ema_alpha;
    for (int i = 0; i < accepted; ++i) g->p[i] = (1.0 - a) * g->p[i] + a;
    if (accepted < drafted) g->p[accepted] = (1.0 - a) * g->p[accepted];
    return MOE_OK;
}

int moe_governor_probabilities(const moe_governor *g, double *p)
{
    if (!g || !p) return MOE_ERR_INVALID_ARG;
    for (size_t i = 0; i < g->p.size(); ++i) p[i] = g->p[i];
    return MOE_OK;
}

int moe_governor_k_accept(const moe_governor *g, int32_t k, double *out)
{
    if (!g || !out || k < 0 || k > g->cfg.k_max) return MOE_ERR_INVALID_ARG;
    *out = k_accept(g, k);
    return MOE_OK;
}

int moe_governor_cycle_time(const moe_governor *g, int32_t k, int32_t n_new, double *t)
{
    if (!g || !t || k < 0 || k > g->cfg.k_max || n_new < 0) return MOE_ERR_INVALID_ARG;
    *t = cycle_time(g, k, n_new);
    return MOE_OK;
}

int moe_governor_evaluate(const moe_governor *g, int32_t k, int32_t n_new, double *theta, double *intensity)
{
    if (!g || k < 0 || k > g->cfg.k_max || n_new < 0) return MOE_ERR_INVALID_ARG;
    const double ka = k_accept(g, k);
    if (theta) *theta = ka / cycle_time(g, k, n_new);
    if (intensity)
        *intensity = n_new == 0 ? std::numeric_limits<double>::infinity() : ka / (n_new * g->cfg.s_expert);
    return MOE_OK;
}

int moe_governor_choose_k(const moe_governor *g, const int32_t *n_new_by_k, int32_t k_slo,
                          int32_t *k_star, double *theta_star)
{
    if (!g || !n_new_by_k || !k_star) return MOE_ERR_INVALID_ARG;
    const int hi = (k_slo > 0 && k_slo < g->cfg.k_max) ? k_slo : g->cfg.k_max;
    if (hi < g->cfg.k_min) return MOE_ERR_INVALID_ARG;
    int best = -1;
    double best_theta = 0.0;
    for (int k = g->cfg.k_min; k <= hi; ++k) {
        if (n_new_by_k[k] < 0) return MOE_ERR_INVALID_ARG;
        const double th = k_accept(g, k) / cycle_time(g, k, n_new_by_k[k]);
        if (best < 0 || th > best_theta) { best = k; best_theta = th; }
    }
    *k_star = best;
    if (theta_star) *theta_star = best_theta;
    return MOE_OK;
}

}  // extern "C"
