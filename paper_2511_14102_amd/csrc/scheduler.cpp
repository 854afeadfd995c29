// Expert Scheduler (paper section 3.3): the Expert Lookahead Buffer and the per-layer expert
// cache (slot tables, lookahead-aware eviction, three-phase prefetch planning, on-demand
// misses) as plain host code behind the C ABI of include/moespeq_sched.h.  It decides; the
// caller copies (moe_expert_copy_async) and uploads the slot tables.
#include <algorithm>
#include <new>
#include <vector>
#include "../../include/moespeq_sched.h"

struct moe_elb {
    int L, k_max, top_k, steps;
    std::vector<int32_t> ids;       // [k_max][L][top_k]
    std::vector<float> conf;
};

struct moe_cache {
    int L, E, C;
    std::vector<int32_t> slot_of;   // [L][E]  -1 = absent
    std::vector<int32_t> expert_in; // [L][C]  -1 = empty
    std::vector<int64_t> last_use;  // [L][E]  clock of the last use (0 = never)
    std::vector<uint8_t> prot;      // [L][E]  named by the current window's ELB
    int64_t clock, hits, misses;
};

namespace {

// slot for a new expert of `layer`: lowest empty slot, else the least recently used resident
// expert for which `evictable` holds (ties: lowest slot); -1 if there is none
template <typename F>
int choose_slot(const moe_cache *c, int layer, F evictable)
{
    const int32_t *in = &c->expert_in[(size_t)layer * c->C];
    for (int s = 0; s < c->C; ++s)
        if (in[s] < 0) return s;
    int best = -1;
    int64_t best_use = 0;
    for (int s = 0; s < c->C; ++s) {
        const int e = in[s];
        if (!evictable(e)) continue;
        const int64_t u = c->last_use[(size_t)layer * c->E + e];
        if (best < 0 || u < best_use) { best = s; best_use = u; }
    }
    return best;
}

moe_fetch install(moe_cache *c, int layer, int expert, int slot)
{
    int32_t *in = &c->expert_in[(size_t)layer * c->C];
    int32_t *so = &c->slot_of[(size_t)layer * c->E];
    moe_fetch f = {layer, expert, slot, in[slot]};
    if (in[slot] >= 0) so[in[slot]] = -1;
    in[slot] = expert;
    so[expert] = slot;
    return f;
}

}  // namespace

extern "C" {

int moe_elb_create(moe_elb **out, int32_t n_layers, int32_t k_max, int32_t top_k)
{
    if (!out || n_layers < 1 || k_max < 1 || k_max > MOE_GOVERNOR_MAX_K || top_k < 1 || top_k > MOE_MAX_TOPK)
        return MOE_ERR_INVALID_ARG;
    moe_elb *e = new (std::nothrow) moe_elb;
    if (!e) return MOE_ERR_HIP;
    e->L = n_layers; e->k_max = k_max; e->top_k = top_k; e->steps = 0;
    e->ids.assign((size_t)k_max * n_layers * top_k, -1);
    e->conf.assign((size_t)k_max * n_layers * top_k, 0.f);
    *out = e;
    return MOE_OK;
}

int moe_elb_destroy(moe_elb *elb) { delete elb; return MOE_OK; }

int moe_elb_reset(moe_elb *elb)
{
    if (!elb) return MOE_ERR_INVALID_ARG;
    elb->steps = 0;
    return MOE_OK;
}

int moe_elb_put_step(moe_elb *elb, int32_t step, const int32_t *ids, const float *conf)
{
    if (!elb || !ids || step != elb->steps || step >= elb->k_max) return MOE_ERR_INVALID_ARG;
    const size_t n = (size_t)elb->L * elb->top_k, o = (size_t)step * n;
    for (size_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= MOE_MAX_EXPERTS) return MOE_ERR_INVALID_ARG;
        elb->ids[o + i] = ids[i];
        elb->conf[o + i] = conf ? conf[i] : 1.f;
    }
    elb->steps = step + 1;
    return MOE_OK;
}

int moe_elb_steps(const moe_elb *elb, int32_t *n_steps)
{
    if (!elb || !n_steps) return MOE_ERR_INVALID_ARG;
    *n_steps = elb->steps;
    return MOE_OK;
}

int moe_elb_entry(const moe_elb *elb, int32_t step, int32_t layer, int32_t *ids, float *conf)
{
    if (!elb || !ids || step < 0 || step >= elb->steps || layer < 0 || layer >= elb->L) return MOE_ERR_INVALID_ARG;
    const size_t o = ((size_t)step * elb->L + layer) * elb->top_k;
    for (int j = 0; j < elb->top_k; ++j) {
        ids[j] = elb->ids[o + j];
        if (conf) conf[j] = elb->conf[o + j];
    }
    return MOE_OK;
}

int moe_cache_create(moe_cache **out, int32_t n_layers, int32_t n_experts, int32_t n_slots)
{
    if (!out || n_layers < 1 || n_experts < 1 || n_experts > MOE_MAX_EXPERTS || n_slots < 1 || n_slots > n_experts)
        return MOE_ERR_INVALID_ARG;
    moe_cache *c = new (std::nothrow) moe_cache;
    if (!c) return MOE_ERR_HIP;
    c->L = n_layers; c->E = n_experts; c->C = n_slots;
    c->slot_of.assign((size_t)n_layers * n_experts, -1);
    c->expert_in.assign((size_t)n_layers * n_slots, -1);
    c->last_use.assign((size_t)n_layers * n_experts, 0);
    c->prot.assign((size_t)n_layers * n_experts, 0);
    c->clock = 0; c->hits = 0; c->misses = 0;
    *out = c;
    return MOE_OK;
}

int moe_cache_destroy(moe_cache *c) { delete c; return MOE_OK; }

int moe_cache_place(moe_cache *c, int32_t layer, int32_t expert, int32_t slot)
{
    if (!c || layer < 0 || layer >= c->L || expert < 0 || expert >= c->E || slot < 0 || slot >= c->C)
        return MOE_ERR_INVALID_ARG;
    if (c->expert_in[(size_t)layer * c->C + slot] >= 0 || c->slot_of[(size_t)layer * c->E + expert] >= 0)
        return MOE_ERR_INVALID_ARG;
    (void)install(c, layer, expert, slot);
    return MOE_OK;
}

int moe_cache_slot_table(const moe_cache *c, int32_t layer, int32_t *slot_of_expert)
{
    if (!c || !slot_of_expert || layer < 0 || layer >= c->L) return MOE_ERR_INVALID_ARG;
    std::copy_n(&c->slot_of[(size_t)layer * c->E], c->E, slot_of_expert);
    return MOE_OK;
}

int moe_cache_use(moe_cache *c, int32_t layer, const int32_t *ids, int32_t n, int32_t *n_hit, int32_t *n_miss)
{
    if (!c || layer < 0 || layer >= c->L || n < 0 || (n > 0 && !ids)) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= c->E) return MOE_ERR_INVALID_ARG;
    const int64_t now = ++c->clock;
    int hit = 0, miss = 0;
    for (int i = 0; i < n; ++i) {
        int64_t &lu = c->last_use[(size_t)layer * c->E + ids[i]];
        if (lu == now) continue;                       // duplicate within this call
        lu = now;
        if (c->slot_of[(size_t)layer * c->E + ids[i]] >= 0) ++hit; else ++miss;
    }
    c->hits += hit; c->misses += miss;
    if (n_hit) *n_hit = hit;
    if (n_miss) *n_miss = miss;
    return MOE_OK;
}

int moe_cache_stats(const moe_cache *c, int64_t *hits, int64_t *misses)
{
    if (!c || !hits || !misses) return MOE_ERR_INVALID_ARG;
    *hits = c->hits; *misses = c->misses;
    return MOE_OK;
}

int moe_cache_end_window(moe_cache *c)
{
    if (!c) return MOE_ERR_INVALID_ARG;
    std::fill(c->prot.begin(), c->prot.end(), (uint8_t)0);
    return MOE_OK;
}

int moe_sched_plan(moe_cache *c, const moe_elb *elb, int32_t phase, int32_t max_fetch, float min_conf,
                   moe_fetch *out, int32_t max_out, int32_t *n_out)
{
    if (!c || !elb || !n_out || elb->L != c->L || max_out < 0 || (max_out > 0 && !out)) return MOE_ERR_INVALID_ARG;
    if (phase != MOE_PHASE_PRIME && phase != MOE_PHASE_GUIDED && phase != MOE_PHASE_SATURATE)
        return MOE_ERR_INVALID_ARG;
    // the largest confidence any entry gives an expert, per layer; -1 = not named
    std::vector<float> best((size_t)c->L * c->E, -1.f);
    for (int s = 0; s < elb->steps; ++s)
        for (int l = 0; l < c->L; ++l)
            for (int j = 0; j < elb->top_k; ++j) {
                const size_t o = ((size_t)s * elb->L + l) * elb->top_k + j;
                const int e = elb->ids[o];
                if (e >= c->E) return MOE_ERR_INVALID_ARG;
                float &b = best[(size_t)l * c->E + e];
                b = std::max(b, elb->conf[o]);
            }
    // candidates in fetch order
    struct Cand { int layer, expert; float conf; };
    std::vector<Cand> cand;
    for (int l = 0; l < c->L; ++l) {
        const size_t first = cand.size();
        for (int e = 0; e < c->E; ++e) {
            const float b = best[(size_t)l * c->E + e];
            if (b < 0.f) continue;
            c->prot[(size_t)l * c->E + e] = 1;
            if (phase == MOE_PHASE_PRIME || c->slot_of[(size_t)l * c->E + e] >= 0) continue;
            if (phase == MOE_PHASE_GUIDED && b < min_conf) continue;
            cand.push_back(Cand{l, e, b});
        }
        if (phase == MOE_PHASE_GUIDED)
            std::stable_sort(cand.begin() + first, cand.end(),
                             [](const Cand &a, const Cand &b) { return a.conf > b.conf; });
    }
    if (phase == MOE_PHASE_GUIDED && (int)cand.size() > std::max(max_fetch, 0)) cand.resize(std::max(max_fetch, 0));
    // dry run of the slot choices on a copy, so that an overflow of `out` changes nothing
    moe_cache trial = *c;
    std::vector<moe_fetch> fetches;
    for (const Cand &k : cand) {
        const uint8_t *prot = &trial.prot[(size_t)k.layer * trial.E];
        const int slot = choose_slot(&trial, k.layer, [&](int e) { return !prot[e]; });
        if (slot < 0) continue;                        // every slot holds an expert the window needs
        fetches.push_back(install(&trial, k.layer, k.expert, slot));
    }
    if ((int)fetches.size() > max_out) return MOE_ERR_WORKSPACE;
    *c = trial;
    std::copy(fetches.begin(), fetches.end(), out);
    *n_out = (int)fetches.size();
    return MOE_OK;
}

int moe_sched_on_demand(moe_cache *c, int32_t layer, const int32_t *missing, int32_t n, moe_fetch *out)
{
    if (!c || layer < 0 || layer >= c->L || n < 0 || (n > 0 && (!missing || !out))) return MOE_ERR_INVALID_ARG;
    if (n > c->C) return MOE_ERR_WORKSPACE;
    std::vector<uint8_t> incoming(c->E, 0);
    for (int i = 0; i < n; ++i) {
        if (missing[i] < 0 || missing[i] >= c->E || incoming[missing[i]] ||
            c->slot_of[(size_t)layer * c->E + missing[i]] >= 0)
            return MOE_ERR_INVALID_ARG;
        incoming[missing[i]] = 1;
    }
    for (int i = 0; i < n; ++i) {
        const int slot = choose_slot(c, layer, [&](int e) { return !incoming[e]; });
        if (slot < 0) return MOE_ERR_WORKSPACE;        // cannot happen with n <= slots
        out[i] = install(c, layer, missing[i], slot);
    }
    return MOE_OK;
}

}  // extern "C"
