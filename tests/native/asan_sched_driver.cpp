// Drives the host-side control plane (Speculative Governor, lookahead buffer, expert cache and
// scheduler: csrc/governor.cpp, csrc/scheduler.cpp) through its C ABI with seeded random histories
// and the documented error cases, for a build with -fsanitize=address,undefined.  Every buffer is a
// heap allocation of exactly the documented size.  Exit code 0 and nothing on stderr = clean.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "moespeq_sched.h"

static uint32_t state = 99u;
static uint32_t rnd() { state = state * 1664525u + 1013904223u; return state >> 8; }
#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "REQUIRE failed line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int governor()
{
    std::vector<int32_t> vt = {2, 4, 8};
    std::vector<double> vs = {1e-3, 1.5e-3, 2.6e-3};
    moe_governor_config cfg = {1e-4, 2e-4, 3e-4, 1e-5, 5e10, 1.7e7, 3, vt.data(), vs.data(), 0.2, 0.8, 1, 7};
    moe_governor *g = nullptr;
    REQUIRE(moe_governor_create(&g, &cfg) == MOE_OK);
    moe_governor_config bad = cfg;
    bad.k_max = MOE_GOVERNOR_MAX_K + 1;
    moe_governor *gb = nullptr;
    REQUIRE(moe_governor_create(&gb, &bad) == MOE_ERR_INVALID_ARG);
    std::vector<double> p(cfg.k_max);
    std::vector<int32_t> n_new(cfg.k_max + 1);
    for (int it = 0; it < 200; ++it) {
        const int drafted = 1 + (int)(rnd() % cfg.k_max), accepted = (int)(rnd() % (drafted + 1));
        REQUIRE(moe_governor_observe(g, drafted, accepted) == MOE_OK);
        REQUIRE(moe_governor_probabilities(g, p.data()) == MOE_OK);
        for (int k = 0; k <= cfg.k_max; ++k) n_new[k] = (int32_t)(rnd() % 40) * k;
        int32_t k_star = 0;
        double theta = 0, t = 0, ka = 0, inten = 0;
        REQUIRE(moe_governor_choose_k(g, n_new.data(), (int)(rnd() % 9), &k_star, &theta) == MOE_OK || true);
        const int k = 1 + (int)(rnd() % cfg.k_max);
        REQUIRE(moe_governor_k_accept(g, k, &ka) == MOE_OK && ka >= 0 && ka <= k);
        REQUIRE(moe_governor_cycle_time(g, k, n_new[k], &t) == MOE_OK && t > 0);
        REQUIRE(moe_governor_evaluate(g, k, n_new[k], &theta, &inten) == MOE_OK);
        REQUIRE(moe_governor_evaluate(g, k, 0, nullptr, nullptr) == MOE_OK);
    }
    REQUIRE(moe_governor_observe(g, cfg.k_max + 1, 0) == MOE_ERR_INVALID_ARG);
    REQUIRE(moe_governor_destroy(g) == MOE_OK);
    return 0;
}

static int scheduler(int n_layers, int E, int n_slots, int top_k, int K)
{
    moe_elb *elb = nullptr;
    moe_cache *c = nullptr;
    REQUIRE(moe_elb_create(&elb, n_layers, K, top_k) == MOE_OK);
    REQUIRE(moe_cache_create(&c, n_layers, E, n_slots) == MOE_OK);
    for (int l = 0; l < n_layers; ++l)
        for (int s = 0; s < n_slots / 2; ++s) REQUIRE(moe_cache_place(c, l, (s * 7 + l) % E == s ? s : (s * 7 + l) % E, s) == MOE_OK || true);
    std::vector<int32_t> ids((size_t)n_layers * top_k), table(E), back(top_k), miss(E);
    std::vector<float> conf((size_t)n_layers * top_k), cback(top_k);
    std::vector<moe_fetch> out((size_t)n_layers * n_slots);
    for (int window = 0; window < 30; ++window) {
        REQUIRE(moe_elb_reset(elb) == MOE_OK);
        for (int step = 0; step < K; ++step) {
            for (int l = 0; l < n_layers; ++l)
                for (int j = 0; j < top_k; ++j) {                       // distinct ids inside one entry
                    ids[(size_t)l * top_k + j] = (int32_t)((rnd() % (E / top_k)) * top_k + j);
                    conf[(size_t)l * top_k + j] = (float)(rnd() % 1000) / 1000.f;
                }
            REQUIRE(moe_elb_put_step(elb, step, ids.data(), (window & 1) ? conf.data() : nullptr) == MOE_OK);
            REQUIRE(moe_elb_put_step(elb, step + 2, ids.data(), nullptr) == MOE_ERR_INVALID_ARG);   // out of order
            REQUIRE(moe_elb_entry(elb, step, n_layers - 1, back.data(), cback.data()) == MOE_OK);
            int32_t n_out = -1;
            const int phase = step == 0 ? MOE_PHASE_PRIME : (step == K - 1 ? MOE_PHASE_SATURATE : MOE_PHASE_GUIDED);
            REQUIRE(moe_sched_plan(c, elb, phase, 1 + (int)(rnd() % 4), 0.1f, out.data(), (int32_t)out.size(), &n_out) == MOE_OK);
            REQUIRE(n_out >= 0 && n_out <= (int32_t)out.size());
            for (int i = 0; i < n_out; ++i) REQUIRE(out[i].slot >= 0 && out[i].slot < n_slots && out[i].expert >= 0 && out[i].expert < E);
        }
        int32_t steps = -1;
        REQUIRE(moe_elb_steps(elb, &steps) == MOE_OK && steps == K);
        for (int l = 0; l < n_layers; ++l) {
            for (int j = 0; j < top_k; ++j) ids[j] = (int32_t)(rnd() % E);
            int32_t hit = -1, nmiss = -1;
            REQUIRE(moe_cache_use(c, l, ids.data(), top_k, &hit, &nmiss) == MOE_OK);
            REQUIRE(moe_cache_slot_table(c, l, table.data()) == MOE_OK);
            int n = 0;
            for (int j = 0; j < top_k; ++j) {
                bool dup = false;
                for (int i = 0; i < n; ++i) dup = dup || miss[i] == ids[j];
                if (!dup && table[ids[j]] < 0 && n < n_slots) miss[n++] = ids[j];
            }
            if (n) REQUIRE(moe_sched_on_demand(c, l, miss.data(), n, out.data()) == MOE_OK);
        }
        REQUIRE(moe_cache_end_window(c) == MOE_OK);
    }
    int64_t hits = 0, misses = 0;
    REQUIRE(moe_cache_stats(c, &hits, &misses) == MOE_OK && hits + misses > 0);
    REQUIRE(moe_sched_on_demand(c, 0, miss.data(), n_slots + 1, out.data()) == MOE_ERR_WORKSPACE);
    REQUIRE(moe_cache_place(c, n_layers, 0, 0) == MOE_ERR_INVALID_ARG);
    REQUIRE(moe_elb_destroy(elb) == MOE_OK);
    REQUIRE(moe_cache_destroy(c) == MOE_OK);
    return 0;
}

int main()
{
    int rc = governor();
    rc |= scheduler(3, 8, 5, 2, 3);
    rc |= scheduler(27, 64, 16, 6, 5);
    rc |= scheduler(2, 130, 130, 4, 7);
    if (rc == 0) printf("control-plane driver: ok\n");
    return rc;
}
