// Draft-pass kernel for a call with ONE token: router, top-k and the SwiGLU FFN of the selected
// experts on group-wise int4 weights in one launch, one workgroup per work item (gfx950).
// (Calls of two to eight tokens run the persistent kernel of draft_int4.hip, longer runs of
// tokens the grouped contraction of draft_prefill.hip.)
//
// Paper section 3.4.3 (one expert-fused kernel instead of per-expert small GEMMs), section 4.1.3
// (4-bit weights in groups along the input dimension), section 3.3.1 (expert id and confidence
// for the lookahead buffer).  The arithmetic is described in draft_common.h, the
// cross-workgroup protocol of the router exchange in draft_int4.hip (the same here).
//
// Work decomposition ("slice fusion").  A work item is (expert, slice of 32 intermediate
// rows): its workgroup computes the 32 gate and 32 up pre-activations (K = H split over the 8
// waves by groups), h = silu(gate) * up, and immediately multiplies h into the 32 matching
// columns of the down projection for all H outputs, adding the partial outputs into y with
// fp32 atomics.  With one token a call has k I / 32 items (400 on the phi shape), about one
// and a half per compute unit: one workgroup per item, two resident per unit, was measured
// as fast or a little faster here than a persistent launch (25.5 against 26.3 us), whose
// continuous stream has nothing to overlap when it is only one or two items long.
#include "draft_common.h"

namespace moespeq {

namespace {

// MT: token capacity of the launch (1, 2, 4 or 8); UPG: 32-code units per group (g / 32); SYM:
// symmetric format (scale blobs, z = 8).  Only MT = 1 is instantiated: calls of two to eight
// tokens run the streaming kernel, longer runs the grouped contraction.
template <int MT, int UPG, bool SYM>
__global__ __launch_bounds__(kThreads, MT <= 2 ? 4 : 2)   // MT <= 2: 4 waves per SIMD, two workgroups per CU
void draft_fused_kernel(const uint16_t *__restrict__ xin, const FusedArgs a)
{
    constexpr int NI = MT < 4 ? MT : 4;          // D rows (tokens) per lane that can be valid
    constexpr int NC = MT > 4 ? 2 : 1;           // lane groups (of 16) whose D rows can be valid
    // tiles a wave keeps in flight (rolling window); no instantiation spills with 8 (two
    // workgroups per CU leave 128 VGPRs per wave for MT <= 2)
    constexpr int kGuWin = 8;
    constexpr int kSzWin = kGuWin / UPG;
    __shared__ double s_part[kWaves];
    __shared__ int32_t s_ids[MOE_MAX_ASSIGN];
    __shared__ float s_w[MOE_MAX_ASSIGN];
    __shared__ float s_conf[MOE_MAX_ASSIGN];
    __shared__ unsigned long long s_mask[MOE_MAX_EXPERTS / 64];
    __shared__ int32_t s_row_a[MT];             // assignment index of each row (token) of this item
    __shared__ int32_t s_cnt;
    __shared__ int32_t s_flag;
    __shared__ double s_few[MT][kLoneWaveTopk];   // few experts: a token's logits for the ranking
    // partial gate/up sums [wave][row block][token in lane group][lane].  With 8 tokens the array
    // (16 KiB) takes the place of the x copy, which is no longer needed by then: the workgroup's LDS
    // then stays under half of a compute unit's, so that two workgroups share a unit.
    constexpr bool kRedOverX = MT >= 8;
    typedef float red_t[4][NI][NC * 16];
    __shared__ float s_red_own[kRedOverX ? 1 : kWaves * 4 * NI * NC * 16];
    __shared__ __attribute__((aligned(16))) uint16_t s_hhi[MT][32], s_hlo[MT][32];
    __shared__ float s_hsum[MT];
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];   // x copy, then its group sums

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = a.T, H = a.H, E = a.E, I = a.I, k = a.k, g = a.g;
    const int n = T * k;
    const int G = H / g;
    const int xstride = H + 8;                   // bf16 elements per token in LDS (+16 B against bank conflicts)
    uint16_t *s_x = reinterpret_cast<uint16_t *>(s_dyn);
    float *s_xsum = reinterpret_cast<float *>(s_dyn + (size_t)MT * xstride * 2);   // [MT][G]
    static_assert(!kRedOverX || sizeof(red_t) * kWaves == (size_t)kWaves * 4 * 4 * 32 * 4, "launcher sizes the dynamic LDS for this");
    red_t *s_red = reinterpret_cast<red_t *>(kRedOverX ? reinterpret_cast<float *>(s_dyn) : s_red_own);
    // routing scratch behind the group sums, used with many experts: logits [MT][E] (fp64), ranks
    const size_t logit_off = ((size_t)MT * xstride * 2 + (size_t)MT * G * 4 + 7) & ~(size_t)7;
    double *s_logit = reinterpret_cast<double *>(s_dyn + logit_off);
    int32_t *s_rank = reinterpret_cast<int32_t *>(s_dyn + logit_off + (size_t)MT * E * 8);
    // ---- 1. router rows owned by this workgroup (fp64 accumulation of exact fp32 products)
    if ((int)blockIdx.x < E) {
        const int nprod = E < (int)gridDim.x ? E : (int)gridDim.x;
        for (int i = blockIdx.x * kThreads + tid; i < T * H; i += nprod * kThreads)
            __hip_atomic_store(&a.y[i], 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int e = blockIdx.x; e < E; e += gridDim.x) {
        const uint16_t *row = a.wr + (size_t)e * H;
        for (int t = 0; t < T; ++t) {
            const uint16_t *xt = xin + (size_t)t * H;
            double acc = 0.0;
            for (int c = tid; c < H / 8; c += kThreads) {
                const u32x4 xv = *reinterpret_cast<const u32x4 *>(xt + c * 8);
                const u32x4 wv = *reinterpret_cast<const u32x4 *>(row + c * 8);
                const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w}, ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc += (double)(bf16_lo(xs[i]) * bf16_lo(ws[i]));     // bf16 x bf16 is exact in fp32
                    acc += (double)(bf16_hi(xs[i]) * bf16_hi(ws[i]));
                }
            }
            acc = wave::sum(acc);
            if (lane == 0) s_part[wave] = acc;
            // every thread's clearing stores have been performed before the workgroup publishes (a
            // workgroup-scope release fence does not imply this wait; it is free here, the loads
            // of the row were issued after the stores and have returned)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid < kReplicas) {                                       // thread r writes replica r
                double l = 0.0;
                for (int w = 0; w < kWaves; ++w) l += s_part[w];
                l += a.bias ? (double)a.bias[e] : 0.0;
                // {logit, tag} leaves as ONE aligned 16-byte agent-scope store and is read with one
                // 16-byte load: a reader sees the tag only together with the logit
                const unsigned long long lb = (unsigned long long)__double_as_longlong(l);
                const u32x4 rec = {(uint32_t)lb, (uint32_t)(lb >> 32), 1u, 0u};
                store16_agent(a.slots + (size_t)tid * a.replica_stride + 2 * ((size_t)t * E + e), rec);
            }
            __syncthreads();
        }
    }
    if (tid == 0) s_flag = 1;
    if (tid < MOE_MAX_EXPERTS / 64) s_mask[tid] = 0ull;
    __syncthreads();

    // ---- 1b. (while the router result travels) stage x in LDS and sum it per group
    const int Ts = T;
    for (int i = tid; i < Ts * (H / 8); i += kThreads) {
        const int t = i / (H / 8), c8 = i % (H / 8);
        const int src = t;
        *reinterpret_cast<u32x4 *>(s_x + t * xstride + c8 * 8) = *reinterpret_cast<const u32x4 *>(xin + (size_t)src * H + c8 * 8);
    }
    __syncthreads();
    for (int i = tid; i < Ts * G * 16; i += kThreads) {       // 16 threads per (token, group)
        const int part = i & 15, tg_ = i >> 4;
        const int t = tg_ / G, gi = tg_ % G;
        const int per = g / 16;                               // 2, 4 or 8 values each
        const uint16_t *src = s_x + t * xstride + gi * g + part * per;
        float v = 0.f;
        for (int j = 0; j < per; ++j) v += __uint_as_float((uint32_t)src[j] << 16);
        v = wave::row_sum(v);
        if (part == 0) s_xsum[t * G + gi] = v;
    }

    // ---- 2. wave t polls the slots of token t (bounded), then selects its top-k
    double sm_logit = -INFINITY;                 // few experts: this lane's logit and rank, for the softmax later
    int sm_rank = MOE_MAX_EXPERTS;
    for (int t = wave; t < T; t += kWaves) {
        double l[4];
        {
            uint32_t spins = 0;
            bool all = false;
            while (!all && ++spins < a.spin_limit) {
                bool mine = true;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = lane + 64 * i;
                    if (e < E) {
                        const u32x4 v = load16_agent(a.slots + (size_t)(blockIdx.x % kReplicas) * a.replica_stride +
                                                     2 * ((size_t)t * E + e));
                        mine = mine && v.z == 1u;
                        l[i] = __longlong_as_double((long long)(((unsigned long long)v.y << 32) | v.x));
                    } else {
                        l[i] = -INFINITY;
                    }
                }
                all = __all(mine);
                if (!all) __builtin_amdgcn_s_sleep(2);
            }
            if (!all) {                          // gave up: the call fails, and says so in the workspace
                if (lane == 0) {
                    s_flag = 0;
                    __hip_atomic_store(a.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                continue;
            }
        }
        if (E <= kLoneWaveTopk) {
            // Rank of every logit in the strict order (larger first, lower index first among equals),
            // so the ranks are a permutation and rank < k selects.  The wave's 64 lanes are P copies of
            // the experts (E2 = E rounded up to a power of two, P = 64 / E2 >= 2): copy q of expert e
            // counts the logits q per .. q per + per - 1 that come before logit e, read from LDS (the
            // lanes of one copy read one address), and the P counts meet through lane exchanges.  Only
            // the selection is on the path to the first weight load; the softmax follows behind the
            // first loads.  (A serial count over all experts in one wave, with the softmax, took 1.1 us
            // for 16 experts: a lone wave issues one dependent instruction every 8 to 16 clocks.)
            if (lane < E) s_few[t][lane] = l[0];
            int E2 = 2;
            while (E2 < E) E2 <<= 1;
            const int P = 64 / E2, per = (E + P - 1) / P;
            const int q = lane / E2, e = lane % E2;
            const double mine = s_few[t][e < E ? e : E - 1];
            int part = 0;
            for (int j = 0; j < per; ++j) {
                const int e2 = q * per + j;
                const double v = s_few[t][e2 < E ? e2 : E - 1];
                part += (int)(e2 < E) & ((int)(v > mine) | ((int)(v == mine) & (int)(e2 < e)));
            }
            for (int d = E2; d < 64; d <<= 1) part += __shfl_xor(part, d, 64);
            if (lane < E) {
                sm_logit = mine;
                sm_rank = part;
                if (part < k) {
                    s_ids[t * k + part] = lane;
                    atomicOr(&s_mask[lane >> 6], 1ull << (lane & 63));
                }
            }
        } else {
            // many experts: the logits go to LDS and all waves rank them (below)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = lane + 64 * i;
                if (e < E) { s_logit[t * E + e] = l[i]; s_rank[t * E + e] = 0; }
            }
        }
    }
    if (E > kLoneWaveTopk) {
        // Ranks in the order (larger first, lower index first among equals), counted by all eight
        // waves, each over its share of the experts; the order is strict, so rank < k selects.  (k
        // rounds of arg-max in the one wave of a token took 5.4 us for 128 experts and k = 8.)
        __syncthreads();
        if (s_flag != 0) {
            for (int t = 0; t < T; ++t) {
                if (E <= 64) wave::count_ranks<1, 4>(s_logit + t * E, s_rank + t * E, E, lane, wave, kWaves);
                else if (E <= 128) wave::count_ranks<2, 4>(s_logit + t * E, s_rank + t * E, E, lane, wave, kWaves);
                else wave::count_ranks<4, 2>(s_logit + t * E, s_rank + t * E, E, lane, wave, kWaves);
            }
        }
        __syncthreads();
        for (int t = wave; t < T && s_flag != 0; t += kWaves) {
            double mine[4];
            int rank[4];
            double mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = lane + 64 * i;
                const bool have = 64 * i < E && e < E;
                mine[i] = have ? s_logit[t * E + e] : -INFINITY;
                rank[i] = have ? s_rank[t * E + e] : MOE_MAX_EXPERTS;
                mx = fmax(mx, mine[i]);
            }
            mx = wave::max(mx);
            // the selection compares the fp64 logits; the softmax values only have to be good to
            // fp32, so they are computed in fp32 from the fp64 differences
            float pe[4], den = 0.f, sel = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pe[i] = rank[i] < MOE_MAX_EXPERTS ? expf((float)(mine[i] - mx)) : 0.f;
                den += pe[i];
            }
            den = wave::sum(den);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pe[i] = pe[i] / den;
                sel += rank[i] < k ? pe[i] : 0.f;
            }
            sel = wave::sum(sel);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (rank[i] < k) {
                    const int e = lane + 64 * i;
                    s_ids[t * k + rank[i]] = e;
                    s_conf[t * k + rank[i]] = pe[i];
                    s_w[t * k + rank[i]] = a.renorm ? pe[i] / sel : pe[i];
                    atomicOr(&s_mask[e >> 6], 1ull << (e & 63));
                }
            }
        }
    }
    __syncthreads();
    const bool ok = s_flag != 0;
    // This workgroup will not look at the slots again: it will draw a ticket.  The tickets are
    // two-level (kTicketGroups first-level counters, then one) so that the returning atomics do
    // not queue up on one address (measured: up to 5 us with one counter).  The compiler turns the
    // atomic (one lane, wave-uniform address) into a form whose result it reads back at once, which
    // waits for everything the drawing wave has in flight.  Where that happens matters: before a
    // barrier the whole workgroup would wait for it, so the ticket is drawn behind the barriers of
    // the item set-up (measured on the phi shape: 25.3 us there, 26.3 right after the first loads,
    // 26.9 before the barrier that ends the gate/up phase; 25.8 and 26.2 with the wait deferred to
    // the kernel's end, when the loads behind the ticket wait for it in the return queue instead).
    uint32_t ticket = 0xffffffffu;
    auto draw_ticket = [&]() {
        if (tid == kThreads - 64)
            ticket = __hip_atomic_fetch_add(a.tickets + blockIdx.x % kTicketGroups, 1u, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
    };
    // ---- 3. this workgroup's item: the u-th distinct expert (ascending id), slice s
    const int nslice = I / 32;
    const int u = blockIdx.x / nslice, slice = blockIdx.x % nslice;
    int expert = -1;
    if (ok) {
        int seen = 0;
        for (int wd = 0; wd < MOE_MAX_EXPERTS / 64 && expert < 0; ++wd) {
            unsigned long long mk = s_mask[wd];
            const int pc = __popcll(mk);
            if (u < seen + pc) {
                for (int r = u - seen; r > 0; --r) mk &= mk - 1ull;
                expert = wd * 64 + __ffsll((long long)mk) - 1;
            }
            seen += pc;
        }
    }
    expert = __builtin_amdgcn_readfirstlane(expert);   // the same in every lane; tell the compiler
    // ---- 3a. the first window of weight loads goes out before anything else of the item is set
    // up: the addresses need only the expert and the slice, and every microsecond of bookkeeping
    // behind them is hidden by their latency.  (Without an expert -- a surplus workgroup -- the
    // addresses are those of expert 0 and the loaded tiles are not used.)
    const int ex = expert >= 0 ? expert : 0;
    const int U = H / 32;
    const int r = lane & 15, c = lane >> 4;                  // MFMA lane coordinates
    const UnpackConsts uk = unpack_consts();
    const char *qb = a.q + (size_t)ex * a.stride_q;
    const char *szb = a.sz + (size_t)ex * a.stride_sz;
    // codes: [gate|up tiles (slice, ku)] then [down tiles (slice, rt)], 64 lanes x 16 B each
    // A tile's address is a wave-uniform base (scalar arithmetic) plus the lane's 16 bytes.
    const int gu0 = slice * U, dn0 = nslice * U + slice * (H / 64);          // first tile of each part
    const uint32_t lane_off = (uint32_t)lane * 16u;
    auto tile_ptr = [&](int tile) {
        return reinterpret_cast<const u32x4 *>(qb + (size_t)tile * 1024 + lane_off);
    };
    // scale/zero: 16 B = the 4 row blocks' (s, z) of lane row r; [gate|up (slice, group)] then
    // [down (group of I, rt)]
    // (symmetric format: 16 B = the 4 row blocks' s of row r for two groups / two row tiles)
    constexpr int kEpl = SYM ? 2 : 1;                        // groups (row tiles) per 16-byte load
    const u32x4 *szgu = reinterpret_cast<const u32x4 *>(szb) + (size_t)slice * (G / kEpl) * 16 + r;
    const u32x4 *szd = reinterpret_cast<const u32x4 *>(szb) + (size_t)nslice * (G / kEpl) * 16 +
                       (size_t)((slice * 32) / g) * (H / (64 * kEpl)) * 16 + r;

    // ---- this wave's tile stream: its gate/up tiles u0 .. u1 (K = H split over the waves by
    // groups), padded to whole windows, then its down row tiles wave, wave + 8, ... (their loads
    // do not depend on h).  A rolling window of kGuWin tiles is in flight.  EVERY load of the
    // stream is unconditional: past the end of a part its address is clamped to the part's
    // last tile.  The compiler counts the loads in flight in program order; a load under a
    // branch makes it wait for all of them wherever it needs one, which empties the window.
    const int nrt = H / 64;
    // (the symmetric format shares a load between two groups / row tiles: whole pairs per wave)
    const int u0 = ((wave * (G / kEpl)) / kWaves) * kEpl * UPG, u1 = (((wave + 1) * (G / kEpl)) / kWaves) * kEpl * UPG;
    const int nt = u1 - u0;
    const int ntp = (nt + kGuWin - 1) / kGuWin * kGuWin;
    const int r0 = ((wave * (nrt / kEpl)) / kWaves) * kEpl, r1 = (((wave + 1) * (nrt / kEpl)) / kWaves) * kEpl;   // this wave's down row tiles
    const int rt_last = r1 > r0 ? r1 - 1 : 0;
    const int g_last = nt > 0 ? (u1 - 1) / UPG : 0;
    auto stream_ptr = [&](int p) -> const u32x4 * {            // p: position in the stream
        const int ku = u0 + p;
        const int rt = r0 + (p - ntp);
        const int gt = gu0 + (ku < u1 ? ku : u1 - 1);
        const int dt = dn0 + (rt < r1 ? rt : rt_last);
        return tile_ptr(p < ntp ? gt : dt);
    };
    // Scale/zero entries are fetched 4 kEpl groups (or row tiles) per load: lane group c
    // takes the 16 bytes of row r of load unit first / kEpl + 4 pk + c, and a lane picks the
    // entry of the group at hand from that lane group with a lane permute.  `first` is a
    // multiple of kEpl everywhere below.
    constexpr int kPerPack = 4 * kEpl;
    constexpr int kSzPacks = (kSzWin + kPerPack - 1) / kPerPack;
    auto gsz_ptr = [&](int first, int pk) {
        const int gi = first / kEpl + 4 * pk + c;
        const int last = g_last / kEpl;
        return szgu + (size_t)(gi < last ? gi : last) * 16;
    };
    // parameters of the j-th group (row tile) after the packs' first one, lane row r
    auto pick = [&](const u32x4 *packs, int j) {
        const u32x4 &v = packs[j / kPerPack];
        const int src = ((j / kEpl) % 4) * 16 + r;
        GroupParams<SYM> p;
        if constexpr (SYM) {
            p.w[0] = (uint32_t)__shfl((int)((j & 1) ? v.z : v.x), src, 64);
            p.w[1] = (uint32_t)__shfl((int)((j & 1) ? v.w : v.y), src, 64);
        } else {
            p.w[0] = (uint32_t)__shfl((int)v.x, src, 64);
            p.w[1] = (uint32_t)__shfl((int)v.y, src, 64);
            p.w[2] = (uint32_t)__shfl((int)v.z, src, 64);
            p.w[3] = (uint32_t)__shfl((int)v.w, src, 64);
        }
        return p;
    };
    // With ONE token all 16 A rows hold that token, so every lane group ends up with the same
    // sums.  Lane group c then finishes row block c only: it loads that block's entry itself
    // (no lane permutes), picks accumulator c and applies scale and zero to one value instead
    // of four.
    constexpr bool kOwnGu = MT == 1;
    using gentry_t = typename std::conditional<SYM, uint16_t, uint32_t>::type;
    const gentry_t *gent_base = reinterpret_cast<const gentry_t *>(szb) + (size_t)slice * G * 64 +
                                (SYM ? r * 8 : r * 4) + c;
    auto gent_load = [&](int gi) -> uint32_t {
        const int t = gi < g_last ? gi : g_last;
        return (uint32_t)__builtin_nontemporal_load(gent_base + (SYM ? (t >> 1) * 128 + (t & 1) * 4 : t * 64));
    };
    const uint32_t cm1 = 0u - (uint32_t)(c & 1), cm2 = 0u - (uint32_t)(c >> 1);
    auto of_my_block = [&](float v0, float v1, float v2, float v3) {   // v_c, chosen with bit masks
        const uint32_t lo = (__float_as_uint(v1) & cm1) | (__float_as_uint(v0) & ~cm1);
        const uint32_t hi = (__float_as_uint(v3) & cm1) | (__float_as_uint(v2) & ~cm1);
        return __uint_as_float((hi & cm2) | (lo & ~cm2));
    };
    u32x4 win[kGuWin], gsz[kSzPacks];
    uint32_t gent[kSzWin] = {};
#pragma unroll
    for (int i = 0; i < kGuWin; ++i) win[i] = __builtin_nontemporal_load(stream_ptr(i));
    if constexpr (kOwnGu) {
#pragma unroll
        for (int j = 0; j < kSzWin; ++j) gent[j] = gent_load(u0 / UPG + j);
    } else {
#pragma unroll
        for (int pk = 0; pk < kSzPacks; ++pk) gsz[pk] = __builtin_nontemporal_load(gsz_ptr(u0 / UPG, pk));
    }
    // the softmax of wave t's token (few experts), off the path to the first weight load: the
    // selection compared the fp64 logits; the softmax values only have to be good to fp32, so they
    // are computed in fp32 from the fp64 differences
    if (E <= kLoneWaveTopk && wave < T && ok) {
        const int t = wave;                      // T <= kWaves: one token per wave
        const double mx = wave::max(sm_logit);
        const float pe = lane < E ? expf((float)(sm_logit - mx)) : 0.f;
        const float conf = pe / wave::sum(pe);
        const bool sel = sm_rank < k;
        const float sel_sum = wave::sum(sel ? conf : 0.f);
        if (sel) {
            s_conf[t * k + sm_rank] = conf;
            s_w[t * k + sm_rank] = a.renorm ? conf / sel_sum : conf;
        }
    }
    // ---- 3b. the rows (tokens) of the item
    if (tid == 0) s_cnt = 0;
    if (tid < MT) s_hsum[tid] = 0.f;
    __syncthreads();
    if (expert >= 0 && wave == 0) {     // rows of the item: assignments with this expert, ascending
        int cnt = 0;
        for (int base = 0; base < n; base += 64) {
            const int aidx = base + lane;
            const bool hit = aidx < n && s_ids[aidx] == expert;
            const unsigned long long b = __ballot(hit);
            if (hit) {
                const int pos = cnt + __popcll(b & ((1ull << lane) - 1ull));
                if (pos < MT) s_row_a[pos] = aidx;
            }
            cnt += __popcll(b);
        }
        if (lane == 0) s_cnt = cnt < MT ? cnt : MT;
    }
    __syncthreads();
    const int cnt = __builtin_amdgcn_readfirstlane(s_cnt);
    draw_ticket();

    if (expert >= 0 && cnt > 0) {
        // A-operand row of this lane: token slot r (slots >= cnt repeat slot 0; their D rows are ignored)
        auto lds_row = [&](int slot) { return s_row_a[slot] / k; };   // where the slot's x was staged
        const uint16_t *xrow = s_x + lds_row(r < cnt ? r : 0) * xstride + c * 8;
        // tokens whose results this lane holds in its D registers: slot 4c + i
        int tok[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int slot = 4 * c + i;
            tok[i] = lds_row(slot < cnt ? slot : 0);
        }

        float tot[4][NI];
        f32x4 acc[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            acc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NI; ++i) tot[d][i] = 0.f;
        }
        float tot1 = 0.f;
        u32x4 xa = *reinterpret_cast<const u32x4 *>(xrow + (nt > 0 ? u0 : 0) * 32);
        // one window of the gate/up part; kGuard: some of its tiles may lie past the wave's run (the
        // padding of the last window) and are skipped.  Full windows carry no per-tile tests.
        auto gu_window = [&](int base, auto guarded) {
            constexpr bool kGuard = decltype(guarded)::value;
            u32x4 gsz_next[kSzPacks];                             // the next window's groups
            uint32_t gent_next[kSzWin];
            if constexpr (kOwnGu) {
#pragma unroll
                for (int j = 0; j < kSzWin; ++j) gent_next[j] = gent_load((u0 + base) / UPG + kSzWin + j);
            } else {
#pragma unroll
                for (int pk = 0; pk < kSzPacks; ++pk)
                    gsz_next[pk] = __builtin_nontemporal_load(gsz_ptr((u0 + base) / UPG + kSzWin, pk));
            }
#pragma unroll
            for (int i = 0; i < kGuWin; ++i) {
                const int pz = base + i, ku = u0 + pz;
                const u32x4 qv = win[i];
                win[i] = __builtin_nontemporal_load(stream_ptr(pz + kGuWin));
                if (!kGuard || ku < u1) {
                    const u32x4 xn = *reinterpret_cast<const u32x4 *>(xrow + (ku + 1 < u1 ? ku + 1 : ku) * 32);
                    acc[0] = mfma(xa, unpack8(qv.x, uk), acc[0]);
                    acc[1] = mfma(xa, unpack8(qv.y, uk), acc[1]);
                    acc[2] = mfma(xa, unpack8(qv.z, uk), acc[2]);
                    acc[3] = mfma(xa, unpack8(qv.w, uk), acc[3]);
                    xa = xn;
                    if (i % UPG == UPG - 1) {                 // end of a group: scale / zero / offset
                        const int gi = ku / UPG;
                        float xs[NI];
#pragma unroll
                        for (int j = 0; j < NI; ++j) xs[j] = s_xsum[tok[j] * G + gi];
                        if constexpr (kOwnGu) {
                            const uint32_t ev = gent[i / UPG];
                            const float sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(ev & 0xffff));
                            const float zp = SYM ? 136.f : (float)__builtin_bit_cast(_Float16, (uint16_t)(ev >> 16)) + 128.f;
                            tot1 += sc * (of_my_block(acc[0][0], acc[1][0], acc[2][0], acc[3][0]) - zp * xs[0]);
#pragma unroll
                            for (int d = 0; d < 4; ++d) acc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
                        } else {
                            const GroupParams<SYM> gp = pick(gsz, i / UPG);
#pragma unroll
                            for (int d = 0; d < 4; ++d) {
                                const float sc = gp.scale(d), zp = gp.zero128(d);
#pragma unroll
                                for (int j = 0; j < NI; ++j) tot[d][j] += sc * (acc[d][j] - zp * xs[j]);
                                acc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
                            }
                        }
                    }
                }
            }
            if constexpr (kOwnGu) {
#pragma unroll
                for (int j = 0; j < kSzWin; ++j) gent[j] = gent_next[j];
            } else {
#pragma unroll
                for (int pk = 0; pk < kSzPacks; ++pk) gsz[pk] = gsz_next[pk];
            }
        };
        {
            int base = 0;
            for (; base + kGuWin <= nt; base += kGuWin) gu_window(base, std::false_type{});
            if (base < ntp) gu_window(base, std::true_type{});
        }
        // the window now holds this wave's first kGuWin down tiles; their scales follow
        constexpr int kDPacks = (kGuWin + kPerPack - 1) / kPerPack;
        auto dsz_ptr = [&](int first, int pk) {
            const int rt = first / kEpl + 4 * pk + c;
            const int last = rt_last / kEpl;
            return szd + (size_t)(rt < last ? rt : last) * 16;
        };
        // With one or two tokens a lane's D registers hold ONE row block of every down tile (its
        // lane group's, see below), so it needs one entry per tile and loads that itself: no lane
        // permutes and no selection among the four entries.
        constexpr bool kOwnEntry = MT <= 2;
        using entry_t = typename std::conditional<SYM, uint16_t, uint32_t>::type;
        const entry_t *dent = reinterpret_cast<const entry_t *>(szb) + (size_t)nslice * G * 64 +
                              (size_t)((slice * 32) / g) * nrt * 64 + (SYM ? r * 8 : r * 4) + c;
        auto dent_load = [&](int rt) -> uint32_t {
            const int t = rt < r1 ? rt : rt_last;
            return (uint32_t)__builtin_nontemporal_load(dent + (SYM ? (t >> 1) * 128 + (t & 1) * 4 : t * 64));
        };
        u32x4 dsz[kDPacks];
        uint32_t dpe[kGuWin] = {};
        if constexpr (kOwnEntry) {
#pragma unroll
            for (int i = 0; i < kGuWin; ++i) dpe[i] = dent_load(r0 + i);
        } else {
#pragma unroll
            for (int pk = 0; pk < kDPacks; ++pk) dsz[pk] = __builtin_nontemporal_load(dsz_ptr(r0, pk));
        }
        if constexpr (kRedOverX) __syncthreads();      // every wave has finished reading x
        if constexpr (kOwnGu) {
            s_red[wave][c][0][r] = tot1;
        } else if (c < NC) {
#pragma unroll
            for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int i = 0; i < NI; ++i) s_red[wave][d][i][c * 16 + r] = tot[d][i];
        }
        __syncthreads();
        // h for (token slot, row): row blocks 0, 1 are gate rows 0-15, 16-31; 2, 3 the matching up rows
        for (int idx = tid; idx < 2 * NI * NC * 16; idx += kThreads) {
            const int lr = idx % (NC * 16), i = (idx / (NC * 16)) % NI, d = idx / (NC * 16 * NI);
            const int slot = 4 * (lr >> 4) + i;
            if (slot < cnt) {
                float gsum = 0.f, usum = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) { gsum += s_red[w][d][i][lr]; usum += s_red[w][d + 2][i][lr]; }
                const float h = gsum / (1.f + expf(-gsum)) * usum;
                const uint16_t hi = f32_to_bf16_rne(h);
                const uint16_t lo = f32_to_bf16_rne(h - __uint_as_float((uint32_t)hi << 16));
                s_hhi[slot][d * 16 + (lr & 15)] = hi;
                s_hlo[slot][d * 16 + (lr & 15)] = lo;
                // sum of the represented h over the slice, per token: the 16 lanes of a
                // (slot, row block) group add up in a fixed order, and the slot's two group
                // sums meet in LDS (two addends commute, so the result does not depend on order)
                float hs = __uint_as_float((uint32_t)hi << 16) + __uint_as_float((uint32_t)lo << 16);
                hs = wave::row_sum(hs);
                if ((lr & 15) == 0) atomicAdd(&s_hsum[slot], hs);
            }
        }
        __syncthreads();

        // ---- down: this wave's row tiles, all H outputs of the slice's 32 columns.
        // The hi and the lo part of h of a token slot are two A rows, so one MFMA yields both
        // products.  With few token slots the 16 A rows have room for more: the tile's row block
        // bl gets its own copy of the h rows at A rows bl * kRs .. (all other rows zero), and the
        // kBpa MFMAs of kBpa row blocks accumulate into ONE D tile, whose lane group(s) bl then
        // hold row block bl.  For one or two tokens that is the whole tile (64 outputs) in one D
        // register pair per token: one 64-lane atomic per token and tile instead of four 16-lane ones.
        constexpr int kBpa = MT <= 2 ? 4 : (MT == 4 ? 2 : 1);    // row blocks per accumulated D tile
        constexpr int kRs = 16 / kBpa;                           // A rows per row block
        constexpr int kLgb = 4 / kBpa;                           // lane groups per row block
        constexpr int ND = MT < 2 ? 1 : 2;                       // token slots per lane
        u32x4 hab[kBpa];
        {
            const int within = r % kRs, slot = (within >> 1) < cnt ? (within >> 1) : 0;
            const u32x4 hv = *reinterpret_cast<const u32x4 *>((within & 1) ? &s_hlo[slot][c * 8] : &s_hhi[slot][c * 8]);
            const bool used = within < 2 * MT;
#pragma unroll
            for (int bl = 0; bl < kBpa; ++bl) {
                const bool on = used && r / kRs == bl;
                hab[bl] = (u32x4){on ? hv.x : 0u, on ? hv.y : 0u, on ? hv.z : 0u, on ? hv.w : 0u};
            }
        }
        const int my_bl = c / kLgb;                              // the row block this lane's D registers hold
        float hsum[ND], rwd[ND];
        int tokd[ND];
        bool live[ND];
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            const int t = 2 * (c % kLgb) + i;
            const int slot = t < cnt ? t : 0;
            const int arow = s_row_a[slot];
            live[i] = t < cnt;
            hsum[i] = s_hsum[slot];
            tokd[i] = arow / k;
            rwd[i] = s_w[arow];
        }
        // one pass over the window: kReload: the slot is refilled with the tile kGuWin further on
        // (clamped, unconditional); the last pass refills nothing
        auto down_pass = [&](int j0, auto reload) {
            constexpr bool kReload = decltype(reload)::value;
            u32x4 dsz_next[kDPacks];
            if (kReload && !kOwnEntry) {
#pragma unroll
                for (int pk = 0; pk < kDPacks; ++pk)
                    dsz_next[pk] = __builtin_nontemporal_load(dsz_ptr(r0 + j0 + kGuWin, pk));
            }
#pragma unroll
            for (int i = 0; i < kGuWin; ++i) {
                const int rt = r0 + j0 + i;
                const u32x4 qv = win[i];
                const uint32_t ev = dpe[i];
                if (kReload) {
                    const int rtn = rt + kGuWin;
                    win[i] = __builtin_nontemporal_load(tile_ptr(dn0 + (rtn < r1 ? rtn : rt_last)));
                    if constexpr (kOwnEntry) dpe[i] = dent_load(rtn);
                }
                if (rt < r1) {
                    GroupParams<SYM> gp;
                    if constexpr (!kOwnEntry) gp = pick(dsz, i);
                    const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                    for (int q = 0; q < 4 / kBpa; ++q) {
                        f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int bl = 0; bl < kBpa; ++bl) o = mfma(hab[bl], unpack8(qw[q * kBpa + bl], uk), o);
                        const int d = q * kBpa + my_bl;          // this lane's row block of the tile
                        float sc, zp;
                        if constexpr (kOwnEntry) {
                            sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(ev & 0xffff));
                            zp = SYM ? 136.f : (float)__builtin_bit_cast(_Float16, (uint16_t)(ev >> 16)) + 128.f;
                        } else {
                            sc = gp.scale(d);
                            zp = gp.zero128(d);
                        }
#pragma unroll
                        for (int j = 0; j < ND; ++j) {
                            if (live[j]) {
                                const float val = sc * ((o[2 * j] + o[2 * j + 1]) - zp * hsum[j]) * rwd[j];
                                __hip_atomic_fetch_add(&a.y[(size_t)tokd[j] * H + rt * 64 + d * 16 + r], val,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
                        }
                    }
                }
            }
            if (kReload && !kOwnEntry) {
#pragma unroll
                for (int pk = 0; pk < kDPacks; ++pk) dsz[pk] = dsz_next[pk];
            }
        };
        const int ndw = r1 - r0;
        int j0 = 0;
        for (; j0 + kGuWin < ndw; j0 += kGuWin) down_pass(j0, std::true_type{});
        down_pass(j0, std::false_type{});
    }

    // ---- 4. last ticket: every workgroup has its logits, put the workspace back to idle
    if (tid == kThreads - 64) {
        const uint32_t grp = blockIdx.x % kTicketGroups;
        const uint32_t members = (gridDim.x - grp + kTicketGroups - 1) / kTicketGroups;
        int last = 0;
        if (ticket == members - 1) {                   // last of its group: second level
            const uint32_t ngroups = gridDim.x < (uint32_t)kTicketGroups ? gridDim.x : (uint32_t)kTicketGroups;
            const uint32_t t2 = __hip_atomic_fetch_add(a.tickets + kTicketGroups, 1u, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
            last = t2 == ngroups - 1;
        }
        s_flag = last;
    }
    __syncthreads();
    if (s_flag) {
        for (int i = tid; i < T * E * kReplicas; i += kThreads)
            __hip_atomic_store(a.slots + (size_t)(i / (T * E)) * a.replica_stride + 2 * (size_t)(i % (T * E)) + 1, 0ull,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid <= kTicketGroups) __hip_atomic_store(a.tickets + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- 5. workgroup 0 reports the routing (and the plan the shared-expert kernels read)
    if (blockIdx.x != 0) return;
    for (int i = tid; i < n; i += kThreads) {
        a.ids_out[i] = ok ? s_ids[i] : -1;
        if (a.conf_out) a.conf_out[i] = ok ? s_conf[i] : 0.f;
    }
    if (a.S > 0) {
        Plan *p = a.plan;
        for (int i = tid; i < n; i += kThreads) { p->perm[i] = i; p->row_live[i] = 0; }
        for (int i = tid; i < a.S * T; i += kThreads) {
            p->row_tok[n + i] = i % T;
            p->row_w[n + i] = 1.f;
            p->row_live[n + i] = 1;
        }
        if (tid < a.S) {
            p->act_expert[tid] = E + tid;
            p->act_off[tid] = n + tid * T;
            p->act_cnt[tid] = T;
            p->act_w0[tid] = (uint64_t)(a.shared + (size_t)tid * a.shared_stride);
            p->act_w1[tid] = 0;
        }
        if (tid == 0) { p->n_active = a.S; p->n_routed_active = 0; p->n_rows = n + a.S * T; p->n_missing = 0; }
    }
}

// dynamic LDS: the bf16 copy of the item's token rows (padded) and their per-group sums; with 8
// rows the partial gate/up sums (8 waves x 4 row blocks x 4 x 32 floats) later take the same place;
// routed call with many experts: fp64 logits and ranks behind them
size_t slice_dynamic_lds(int MT, int H, int g, int E, bool routed)
{
    size_t lds = (size_t)MT * (H + 8) * 2 + (size_t)MT * (H / g) * 4;
    if (routed && E > kLoneWaveTopk) lds = ((lds + 7) & ~(size_t)7) + (size_t)MT * E * 12;
    if (MT >= 8 && lds < (size_t)kWaves * 4 * 4 * 32 * 4) lds = (size_t)kWaves * 4 * 4 * 32 * 4;
    return lds;
}

template <int MT, bool SYM>
void launch_slice_t(const uint16_t *x, const FusedArgs &a, hipStream_t st, int n_groups_of_slices)
{
    const dim3 grid(n_groups_of_slices * (a.I / 32)), block(kThreads);
    const size_t lds = slice_dynamic_lds(MT, a.H, a.g, a.E, true);
    if (a.g == 32) launch_with_lds(draft_fused_kernel<MT, 1, SYM>, grid, block, lds, st, x, a);
    else if (a.g == 64) launch_with_lds(draft_fused_kernel<MT, 2, SYM>, grid, block, lds, st, x, a);
    else launch_with_lds(draft_fused_kernel<MT, 4, SYM>, grid, block, lds, st, x, a);
}

}  // namespace

// one token: router inside the launch, one workgroup per (selected expert, slice)
void launch_draft_one_token(const Shape &s, const DraftFusedArgs &d, hipStream_t st)
{
    const FusedArgs a = fused_args(s, d);
    const uint16_t *x = (const uint16_t *)d.x;
    const int experts = a.E < a.k ? a.E : a.k;
    if (d.symmetric) launch_slice_t<1, true>(x, a, st, experts);
    else launch_slice_t<1, false>(x, a, st, experts);
}

int draft_one_token_resident(const Shape &s, const DraftFusedArgs &d, int n_cu)
{
    const size_t lds = slice_dynamic_lds(1, s.H, s.g, s.E, true);
    int per = 0;
    auto ask = [&](auto kernel) { per = resident_per_cu(kernel, kThreads, lds); };
    if (d.symmetric) {
        if (s.g == 32) ask(draft_fused_kernel<1, 1, true>);
        else if (s.g == 64) ask(draft_fused_kernel<1, 2, true>);
        else ask(draft_fused_kernel<1, 4, true>);
    } else {
        if (s.g == 32) ask(draft_fused_kernel<1, 1, false>);
        else if (s.g == 64) ask(draft_fused_kernel<1, 2, false>);
        else ask(draft_fused_kernel<1, 4, false>);
    }
    return per * n_cu;
}

bool draft_one_token_fits(const Shape &s)
{
    return slice_dynamic_lds(1, s.H, s.g, s.E, true) <= (size_t)(160 - 20) * 1024;
}

}  // namespace moespeq
