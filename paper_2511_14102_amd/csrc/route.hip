// Router, top-k, softmax weights, token->expert histogram / permutation, execution plan and
// expert union kernels (gfx950).
//
// Paper section 2.1: the router turns a token's hidden state into a distribution over the
// experts and the top-k experts are selected, weighted by their scores.  Section 3.4.2: the
// gate stays 16-bit in the draft model because routing errors corrupt the lookahead, so the
// logits here are accumulated in fp64 (products of two bf16 values are exact), which keeps
// the selected ids identical to an exact evaluation unless two logits agree to ~1e-13.
// Section 3.4.4: assignments are regrouped per expert.  Section 2.3 / 3.2.2: union of the
// experts of a window and the part of it that is not resident.
#include "plan.h"
#include "wave.h"

namespace moespeq {

namespace {

constexpr int kRouteThreads = 1024;

// One workgroup per token: logits of all experts (one wave per expert row at a time), ranks of
// the logits counted by all waves, then wave 0 writes the k selected experts in rank order with
// their softmax weights.
// kAgent: the results are stored at agent scope (another workgroup of the same launch reads them).
template <bool kAgent, typename V>
__device__ inline void put(V *p, V v) {
    if (kAgent) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool kAgent, typename V>
__device__ inline V get(const V *p) {
    return kAgent ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
}

template <bool kAgent>
__device__ inline void route_token(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr,
                                   const float *__restrict__ bias, int H, int E, int k, int renorm,
                                   int32_t *__restrict__ ids, float *__restrict__ w, float *__restrict__ conf)
{
    __shared__ double s_logit[MOE_MAX_EXPERTS];
    __shared__ int32_t s_rank[MOE_MAX_EXPERTS];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwave = kRouteThreads / 64;
    const uint16_t *xt = x + (size_t)t * H;
    const int chunks = H / 8;

    for (int e = wave; e < E; e += nwave) {
        const uint16_t *row = wr + (size_t)e * H;
        // eight independent partial sums instead of one chain of dependent fp64 additions; the
        // products are exact in fp32 (bf16 x bf16).  (The loop is bound by the instruction rate of
        // the one compute unit a token's workgroup runs on: batching the loads did not help.)
        double part[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
        for (int c = lane; c < chunks; c += 64) {
            uint4 xv = *reinterpret_cast<const uint4 *>(xt + c * 8);
            uint4 wv = *reinterpret_cast<const uint4 *>(row + c * 8);
            const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w};
            const uint32_t ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                part[2 * i] += (double)(__uint_as_float(xs[i] << 16) * __uint_as_float(ws[i] << 16));
                part[2 * i + 1] += (double)(__uint_as_float(xs[i] & 0xffff0000u) * __uint_as_float(ws[i] & 0xffff0000u));
            }
        }
        double acc = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
        acc = wave::sum(acc);
        if (lane == 0) { s_logit[e] = acc + (bias ? (double)bias[e] : 0.0); s_rank[e] = 0; }
    }

    __syncthreads();
    // Rank of every logit under (larger first, lower index first among equals), counted by all
    // sixteen waves, each over its share of the experts (one wave alone needs microseconds for a
    // serial selection: about 16 clocks per instruction, and the count grows with E).  The order is
    // strict, so the ranks are a permutation and rank < k is the selection.
    wave::count_ranks(s_logit, s_rank, E, lane, wave, nwave);
    __syncthreads();
    if (wave != 0) return;                 // (the caller's next barrier is reached by all waves)
    double mine[4], pe[4];
    int rank[4];
    double mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        const bool have = 64 * i < E && e < E;
        mine[i] = have ? s_logit[e] : -INFINITY;
        rank[i] = have ? s_rank[e] : MOE_MAX_EXPERTS;
        mx = fmax(mx, mine[i]);
    }
    mx = wave::max(mx);
    double den = 0.0, sel = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pe[i] = rank[i] < MOE_MAX_EXPERTS ? exp(mine[i] - mx) : 0.0;
        den += pe[i];
    }
    den = wave::sum(den);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pe[i] = pe[i] / den;
        sel += rank[i] < k ? pe[i] : 0.0;
    }
    sel = wave::sum(sel);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (rank[i] < k) {
            const size_t o = (size_t)t * k + rank[i];
            put<kAgent>(&ids[o], (int32_t)(lane + 64 * i));
            const float c = (float)pe[i];
            if (conf) put<kAgent>(&conf[o], c);
            put<kAgent>(&w[o], renorm ? (float)(pe[i] / sel) : c);
        }
    }
}

__global__ __launch_bounds__(kRouteThreads)
void route_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr,
                  const float *__restrict__ bias, int H, int E, int k, int renorm,
                  int32_t *__restrict__ ids, float *__restrict__ w, float *__restrict__ conf)
{
    route_token<false>(x, wr, bias, H, E, k, renorm, ids, w, conf);
}

// count / off / perm for n <= MOE_MAX_ASSIGN assignments over E experts; one workgroup of at least
// 256 threads, results in `count`, `off`, `perm` (global or shared memory), `ids` in LDS.
// Thread a owns assignment a: counts by LDS atomics, offsets by a scan in wave 0 (four experts per
// lane), and the place of a inside its expert is the number of earlier assignments with the same
// expert, counted over broadcast reads of ids (ascending a inside an expert: stable).  The loops
// of the first version (thread e scanning all assignments and all smaller experts, one dependent
// LDS read per step) took 12 us for 64 assignments over 128 experts.
__device__ inline void histogram_perm(const int32_t *ids, int n, int E, int32_t *count,
                                      int32_t *off, int32_t *perm, int32_t *s_count)
{
    __shared__ int32_t s_excl[MOE_MAX_EXPERTS + 1];
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += blockDim.x) s_count[e] = 0;
    __syncthreads();
    const int my_e = tid < n ? ids[tid] : -1;
    if (tid < n) atomicAdd(&s_count[my_e], 1);
    __syncthreads();
    if (tid < 64) {
        int c[4], sum = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = 4 * tid + i;
            c[i] = e < E ? s_count[e] : 0;
            sum += c[i];
        }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int v = __shfl_up(incl, d, 64);
            if (tid >= d) incl += v;
        }
        int base = incl - sum;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = 4 * tid + i;
            if (e < E) s_excl[e] = base;
            base += c[i];
        }
        if (tid == 0) s_excl[E] = n;
    }
    __syncthreads();
    for (int e = tid; e <= E; e += blockDim.x) {
        off[e] = s_excl[e];
        if (e < E) count[e] = s_count[e];
    }
    if (tid < n) {
        int before = 0;
        for (int a = 0; a < n; a += 8) {
            int v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = ids[a + j < n ? a + j : n - 1];       // the same address in every lane
#pragma unroll
            for (int j = 0; j < 8; ++j) before += (int)(a + j < tid) & (int)(v[j] == my_e);
        }
        perm[s_excl[my_e] + before] = tid;
    }
    __syncthreads();
}

__global__ __launch_bounds__(256)
void perm_kernel(const int32_t *__restrict__ ids, int n, int E, int32_t *count, int32_t *off,
                 int32_t *perm)
{
    __shared__ int32_t s_ids[MOE_MAX_ASSIGN];
    __shared__ int32_t s_count[MOE_MAX_EXPERTS];
    for (int a = threadIdx.x; a < n; a += blockDim.x) s_ids[a] = ids[a];
    __syncthreads();
    histogram_perm(s_ids, n, E, count, off, perm, s_count);
}

// Plan that runs only the S shared experts over T tokens (rows n .. n + S T, n = T k routed rows
// that stay dead): what the draft kernel leaves for the shared-expert kernels, for callers that
// route elsewhere.
__global__ __launch_bounds__(256)
void shared_plan_kernel(Plan *__restrict__ p, int T, int k, int S, int E, const char *shared, size_t shared_stride)
{
    const int n = T * k, tid = threadIdx.x;
    for (int i = tid; i < n; i += 256) { p->perm[i] = i; p->row_live[i] = 0; }
    for (int i = tid; i < S * T; i += 256) {
        p->row_tok[n + i] = i % T;
        p->row_w[n + i] = 1.f;
        p->row_live[n + i] = 1;
    }
    if (tid < S) {
        p->act_expert[tid] = E + tid;
        p->act_off[tid] = n + tid * T;
        p->act_cnt[tid] = T;
        p->act_w0[tid] = (uint64_t)(shared + (size_t)tid * shared_stride);
        p->act_w1[tid] = 0;
    }
    if (tid == 0) { p->n_active = S; p->n_routed_active = 0; p->n_rows = n + S * T; p->n_missing = 0; }
}

// Builds the execution plan: histogram / permutation, the list of experts to run (shared
// experts at active indices [0, S), then present routed experts ascending), their weight
// pointers and row ranges, the per-row token / weight / live flags, and the missing list.
template <bool kAgent>
__device__ inline void plan_body(Plan *__restrict__ plan, int T, int E, int k, int S, int mode,
                 const char *w0, size_t stride0, const char *w1, size_t stride1,
                 const int32_t *__restrict__ slot_of_expert,
                 const char *shared, size_t shared_stride, int flags,
                 int32_t *ids_out, float *conf_out, int32_t *missing, int32_t *n_missing)
{
    __shared__ int32_t s_ids[MOE_MAX_ASSIGN];
    __shared__ int32_t s_count[MOE_MAX_EXPERTS];
    __shared__ int32_t s_slot[MOE_MAX_EXPERTS];
    __shared__ unsigned char s_listed[MOE_MAX_EXPERTS];
    __shared__ int32_t s_off[MOE_MAX_EXPERTS + 1];     // offsets and permutation stay in LDS for the
    __shared__ int32_t s_perm[MOE_MAX_ASSIGN];         // steps below; the plan gets a copy
    __shared__ int32_t s_nact, s_nmiss;
    const int n = T * k;
    const bool only_listed = (flags & MOE_VERIFY_ONLY_LISTED) != 0;

    for (int a = threadIdx.x; a < n; a += blockDim.x) {
        int id = get<kAgent>(&plan->ids[a]);
        s_ids[a] = id;
        if (ids_out) ids_out[a] = id;
        if (conf_out) conf_out[a] = get<kAgent>(&plan->conf[a]);
    }
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        s_slot[e] = mode == 0 ? e : slot_of_expert[e];
        s_listed[e] = only_listed ? 0 : 1;
    }
    __syncthreads();
    if (only_listed) {
        int nin = *n_missing;
        nin = nin < 0 ? 0 : (nin > E ? E : nin);
        for (int i = threadIdx.x; i < nin; i += blockDim.x) {
            int e = missing[i];
            if (e >= 0 && e < E) s_listed[e] = 1;
        }
    }
    __syncthreads();
    histogram_perm(s_ids, n, E, plan->count, s_off, s_perm, s_count);
    for (int e = threadIdx.x; e <= E; e += blockDim.x) plan->off[e] = s_off[e];
    for (int i = threadIdx.x; i < n; i += blockDim.x) plan->perm[i] = s_perm[i];

    // shared experts: active slots [0, S), rows T*k + s*T + t
    for (int i = threadIdx.x; i < S * T; i += blockDim.x) {
        plan->row_tok[n + i] = i % T;
        plan->row_w[n + i] = 1.f;
        plan->row_live[n + i] = only_listed ? 0 : 1;
    }
    if ((int)threadIdx.x < S) {
        int s = threadIdx.x;
        plan->act_expert[s] = E + s;
        plan->act_off[s] = n + s * T;
        plan->act_cnt[s] = only_listed ? 0 : T;
        plan->act_w0[s] = (uint64_t)(shared + (size_t)s * shared_stride);
        plan->act_w1[s] = 0;
    }
    // routed experts: ordered compaction, 64 experts per step, by wave 0
    if (threadIdx.x < 64) {
        int nact = S, nmiss = 0;
        for (int base = 0; base < E; base += 64) {
            int e = base + threadIdx.x;
            bool used = e < E && s_count[e] > 0 && s_listed[e];
            bool present = used && s_slot[e] >= 0;
            bool absent = used && s_slot[e] < 0;
            unsigned long long bp = __ballot(present), ba = __ballot(absent);
            unsigned long long below = (1ull << threadIdx.x) - 1ull;
            if (present) {
                int u = nact + __popcll(bp & below);
                int slot = s_slot[e];
                plan->act_expert[u] = e;
                plan->act_off[u] = s_off[e];
                plan->act_cnt[u] = s_count[e];
                plan->act_w0[u] = (uint64_t)(w0 + (size_t)slot * stride0);
                plan->act_w1[u] = w1 ? (uint64_t)(w1 + (size_t)slot * stride1) : 0;
            }
            if (absent) missing[nmiss + __popcll(ba & below)] = e;
            nact += __popcll(bp);
            nmiss += __popcll(ba);
        }
        if (threadIdx.x == 0) { s_nact = nact; s_nmiss = nmiss; }
    }
    __syncthreads();
    for (int pos = threadIdx.x; pos < n; pos += blockDim.x) {
        int a = s_perm[pos];
        int e = s_ids[a];
        plan->row_tok[pos] = a / k;
        plan->row_w[pos] = get<kAgent>(&plan->w[a]);
        plan->row_live[pos] = (s_listed[e] && s_slot[e] >= 0) ? 1 : 0;
    }
    if (threadIdx.x == 0) {
        plan->n_active = s_nact;
        plan->n_routed_active = s_nact - S;
        plan->n_rows = n + S * T;
        plan->n_missing = s_nmiss;
        if (n_missing) *n_missing = s_nmiss;
    }
}

struct PlanKernelArgs {
    Plan *plan; int T, E, k, S, mode;
    const char *w0; size_t stride0; const char *w1; size_t stride1;
    const int32_t *slot_of_expert; const char *shared; size_t shared_stride; int flags;
    int32_t *ids_out; float *conf_out; int32_t *missing; int32_t *n_missing;
};

__global__ __launch_bounds__(256)
void plan_kernel(const PlanKernelArgs a)
{
    plan_body<false>(a.plan, a.T, a.E, a.k, a.S, a.mode, a.w0, a.stride0, a.w1, a.stride1, a.slot_of_expert,
                     a.shared, a.shared_stride, a.flags, a.ids_out, a.conf_out, a.missing, a.n_missing);
}

// Router and plan in one launch (the verify call).  Workgroup (b, t) reduces the router rows of
// experts 16 b .. 16 b + 15 for token t, one row per wave, and stores the fp64 logits at agent
// scope; the workgroup that arrives last for its token (a counter per token) has all of the
// token's logits in reach, ranks them, forms the softmax weights and stores ids / weights /
// confidences; the workgroup that arrives last of all builds the plan.  All counters live in the
// workspace, are zero between launches and are put back to zero by the last arrival.  (One
// workgroup per token computing all E rows took 25 us for 128 experts: the instruction rate of
// the one compute unit a token ran on.)
constexpr int kRouteBlock = kRouteThreads / 64;          // experts per workgroup: one per wave

__global__ __launch_bounds__(kRouteThreads)
void route_plan_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr,
                       const float *__restrict__ bias, int H, int renorm, const PlanKernelArgs a,
                       double *logits, uint32_t *token_arrivals, uint32_t *arrivals)
{
    __shared__ double s_logit[MOE_MAX_EXPERTS];
    __shared__ int32_t s_rank[MOE_MAX_EXPERTS];
    __shared__ int s_last;
    const int t = blockIdx.y, E = a.E, k = a.k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nblk = gridDim.x;
    const int e = blockIdx.x * kRouteBlock + wave;
    if (e < E) {
        const uint16_t *xt = x + (size_t)t * H, *row = wr + (size_t)e * H;
        // eight independent partial sums instead of one chain of dependent fp64 additions; the
        // products are exact in fp32 (bf16 x bf16)
        double part[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
        for (int c = lane; c < H / 8; c += 64) {
            uint4 xv = *reinterpret_cast<const uint4 *>(xt + c * 8);
            uint4 wv = *reinterpret_cast<const uint4 *>(row + c * 8);
            const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w};
            const uint32_t ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                part[2 * i] += (double)(__uint_as_float(xs[i] << 16) * __uint_as_float(ws[i] << 16));
                part[2 * i + 1] += (double)(__uint_as_float(xs[i] & 0xffff0000u) * __uint_as_float(ws[i] & 0xffff0000u));
            }
        }
        double acc = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
        acc = wave::sum(acc);
        if (lane == 0) {
            acc += bias ? (double)bias[e] : 0.0;
            if (nblk > 1) __hip_atomic_store(&logits[(size_t)t * E + e], acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else { s_logit[e] = acc; s_rank[e] = 0; }
        }
    }
    if (nblk > 1) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this thread's stores have been performed
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t n = __hip_atomic_fetch_add(&token_arrivals[t], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = n == (uint32_t)nblk - 1;
            if (s_last) __hip_atomic_store(&token_arrivals[t], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!s_last) return;
        for (int i = threadIdx.x; i < E; i += kRouteThreads) {
            s_logit[i] = __hip_atomic_load(&logits[(size_t)t * E + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_rank[i] = 0;
        }
    }
    __syncthreads();
    // Rank of every logit under (larger first, lower index first among equals), counted by all
    // sixteen waves, each over its share of the experts; the order is strict, so the ranks are a
    // permutation and rank < k is the selection.
    wave::count_ranks(s_logit, s_rank, E, lane, wave, kRouteThreads / 64);
    __syncthreads();
    if (wave == 0) {
        double mine[4], pe[4];
        int rank[4];
        double mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ei = lane + 64 * i;
            const bool have = 64 * i < E && ei < E;
            mine[i] = have ? s_logit[ei] : -INFINITY;
            rank[i] = have ? s_rank[ei] : MOE_MAX_EXPERTS;
            mx = fmax(mx, mine[i]);
        }
        mx = wave::max(mx);
        double den = 0.0, sel = 0.0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pe[i] = rank[i] < MOE_MAX_EXPERTS ? exp(mine[i] - mx) : 0.0;
            den += pe[i];
        }
        den = wave::sum(den);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pe[i] = pe[i] / den;
            sel += rank[i] < k ? pe[i] : 0.0;
        }
        sel = wave::sum(sel);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (rank[i] < k) {
                const size_t o = (size_t)t * k + rank[i];
                put<true>(&a.plan->ids[o], (int32_t)(lane + 64 * i));
                const float c = (float)pe[i];
                put<true>(&a.plan->conf[o], c);
                put<true>(&a.plan->w[o], renorm ? (float)(pe[i] / sel) : c);
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this thread's stores have been performed
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t n = __hip_atomic_fetch_add(arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = n == gridDim.y - 1;
        if (s_last) __hip_atomic_store(arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    plan_body<true>(a.plan, a.T, a.E, a.k, a.S, a.mode, a.w0, a.stride0, a.w1, a.stride1, a.slot_of_expert,
                    a.shared, a.shared_stride, a.flags, a.ids_out, a.conf_out, a.missing, a.n_missing);
}

// Union of expert ids: bitmask in shared memory, then ordered compaction by one wave.
__global__ __launch_bounds__(256)
void union_kernel(const int32_t *__restrict__ ids, int n_ids, int E,
                  const int32_t *__restrict__ slot, uint64_t *mask, int32_t *list,
                  int32_t *n_list, int32_t *missing, int32_t *n_missing)
{
    __shared__ unsigned int s_bits[MOE_MAX_EXPERTS / 32];
    if (threadIdx.x < MOE_MAX_EXPERTS / 32) s_bits[threadIdx.x] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n_ids; i += blockDim.x) {
        int e = ids[i];
        if (e >= 0 && e < E) atomicOr(&s_bits[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
    if (threadIdx.x >= 64) return;
    const int words = (E + 63) / 64;
    if ((int)threadIdx.x < words)
        mask[threadIdx.x] = (uint64_t)s_bits[2 * threadIdx.x] | ((uint64_t)s_bits[2 * threadIdx.x + 1] << 32);
    int nl = 0, nm = 0;
    for (int base = 0; base < E; base += 64) {
        int e = base + threadIdx.x;
        bool in = e < E && ((s_bits[e >> 5] >> (e & 31)) & 1u);
        bool miss = in && slot && slot[e] < 0;
        unsigned long long bi = __ballot(in), bm = __ballot(miss);
        unsigned long long below = (1ull << threadIdx.x) - 1ull;
        if (in) list[nl + __popcll(bi & below)] = e;
        if (miss) missing[nm + __popcll(bm & below)] = e;
        nl += __popcll(bi);
        nm += __popcll(bm);
    }
    if (threadIdx.x == 0) { *n_list = nl; *n_missing = nm; }
}

}  // namespace

void launch_route(const Shape &s, const void *x, const void *wr, const float *bias,
                  int32_t *ids, float *w, float *conf, hipStream_t st)
{
    launch(route_kernel, dim3(s.T), dim3(kRouteThreads), 0, st,
                       (const uint16_t *)x, (const uint16_t *)wr, bias, s.H, s.E, s.k, s.renorm,
                       ids, w, conf);
}

void launch_perm(const Shape &s, const int32_t *ids, int32_t *count, int32_t *off,
                 int32_t *perm, hipStream_t st)
{
    launch(perm_kernel, dim3(1), dim3(256), 0, st, ids, s.T * s.k, s.E, count, off, perm);
}

static PlanKernelArgs plan_kernel_args(const Shape &s, const PlanArgs &a)
{
    PlanKernelArgs k;
    k.plan = a.plan; k.T = s.T; k.E = s.E; k.k = s.k; k.S = s.S; k.mode = a.mode;
    k.w0 = (const char *)a.w0; k.stride0 = a.stride0; k.w1 = (const char *)a.w1; k.stride1 = a.stride1;
    k.slot_of_expert = a.slot_of_expert; k.shared = (const char *)a.shared; k.shared_stride = a.shared_stride;
    k.flags = a.flags; k.ids_out = a.ids_out; k.conf_out = a.conf_out; k.missing = a.missing; k.n_missing = a.n_missing;
    return k;
}

void launch_plan(const Shape &s, const PlanArgs &a, hipStream_t st)
{
    launch(plan_kernel, dim3(1), dim3(256), 0, st, plan_kernel_args(s, a));
}

void launch_route_plan(const Shape &s, const void *x, const void *wr, const float *bias, const PlanArgs &a,
                       double *logits, uint32_t *token_arrivals, uint32_t *arrivals, hipStream_t st)
{
    const dim3 grid((s.E + kRouteBlock - 1) / kRouteBlock, s.T);
    launch(route_plan_kernel, grid, dim3(kRouteThreads), 0, st, (const uint16_t *)x, (const uint16_t *)wr,
           bias, s.H, s.renorm, plan_kernel_args(s, a), logits, token_arrivals, arrivals);
}

void launch_shared_plan(const Shape &s, Plan *plan, const void *shared, size_t shared_stride, hipStream_t st)
{
    launch(shared_plan_kernel, dim3(1), dim3(256), 0, st, plan, s.T, s.k, s.S, s.E, (const char *)shared, shared_stride);
}

void launch_union(const int32_t *ids, int n_ids, int E, const int32_t *slot,
                  uint64_t *mask, int32_t *list, int32_t *n_list,
                  int32_t *missing, int32_t *n_missing, hipStream_t st)
{
    launch(union_kernel, dim3(1), dim3(256), 0, st, ids, n_ids, E, slot, mask, list,
                       n_list, missing, n_missing);
}

}  // namespace moespeq
