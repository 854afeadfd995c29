// Host side of the C ABI declared in include/moespeq.h: argument validation, workspace
// carve-up and kernel sequencing.  No device memory is allocated here and no call waits for
// the device (except the documented MOE_VERIFY_STRICT mode).
#include <string.h>
#include <new>
#include <utility>
#include <vector>
#include "plan.h"

struct moe_ctx {
    int device;
    int n_cu;
    void *scratch;          // this device's address of the static scratch array
    uint32_t spin_limit;    // polls of the router result before a draft workgroup gives up
    char arch[64];
    char hip_error[128];
    bool profiling;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs[MOE_KERNEL_COUNT];   // recorded, not yet read
    std::vector<hipEvent_t> free_events;
};

// Scratch of the allocation-free draft call (moe_draft_layer_int4_noalloc).  Every GPU the library
// runs on holds its own copy of the array, at its own address, until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call
// returned (moe_create asks once per context, with the context's device current).
constexpr size_t kStaticScratchBytes = (size_t)2 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace moespeq {

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

WsLayout ws_layout(const moe_layer_desc &d, int T)
{
    WsLayout L;
    const size_t n = (size_t)T * d.top_k, rows = n + (size_t)T * d.n_shared;
    size_t o = 0;
    L.tickets = o; o += kWsHeadBytes;
    // replicas are skewed by 256 bytes so that they do not all map to the same memory channel
    L.slot_replica_bytes = align256((size_t)MOE_MAX_DRAFT_TOKENS * d.n_experts * 16) + 256;
    L.slots = o;   o += kDraftSlotReplicas * L.slot_replica_bytes;
    L.plan = o;   o += align256(sizeof(Plan));
    L.vlogits = o; o += align256((size_t)MOE_MAX_TOKENS * d.n_experts * 8);   // verify router: fp64 logits [T, E]
    L.hb = o;     o += align256(rows * d.inter * 2);
    L.hb_lo = o;  o += align256(rows * d.inter * 2);
    L.obuf = o;   o += align256(rows * d.hidden * 4);
    L.total = o;
    return L;
}

static bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

static int check_desc(const moe_layer_desc *d)
{
    if (!d) return MOE_ERR_INVALID_ARG;
    if (d->hidden < 64 || d->hidden % 64 || d->inter < 64 || d->inter % 64) return MOE_ERR_INVALID_ARG;
    if (d->hidden > (1 << 16) || d->inter > (1 << 17)) return MOE_ERR_INVALID_ARG;
    if (d->n_experts < 1 || d->n_experts > MOE_MAX_EXPERTS) return MOE_ERR_INVALID_ARG;
    if (d->top_k < 1 || d->top_k > MOE_MAX_TOPK || d->top_k > d->n_experts) return MOE_ERR_INVALID_ARG;
    if (d->n_shared < 0 || d->n_shared > MOE_MAX_SHARED) return MOE_ERR_INVALID_ARG;
    const int g = d->group_size;
    if (g != 32 && g != 64 && g != 128) return MOE_ERR_INVALID_ARG;
    if (d->hidden % g || d->inter % g) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

static int check_tokens(const moe_layer_desc *d, int T, int maxT)
{
    if (T < 1 || T > maxT || T * d->top_k > MOE_MAX_ASSIGN) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

static Shape make_shape(const moe_layer_desc *d, int T)
{
    Shape s;
    s.T = T; s.H = d->hidden; s.E = d->n_experts; s.I = d->inter; s.k = d->top_k;
    s.S = d->n_shared; s.g = d->group_size; s.renorm = d->renormalize ? 1 : 0;
    return s;
}

static int hip_status(moe_ctx *ctx, hipError_t e)
{
    if (e == hipSuccess) return MOE_OK;
    if (ctx) {
        strncpy(ctx->hip_error, hipGetErrorName(e), sizeof(ctx->hip_error) - 1);
        ctx->hip_error[sizeof(ctx->hip_error) - 1] = 0;
    }
    return MOE_ERR_HIP;
}

thread_local LaunchTiming g_launch_timing = {nullptr, nullptr};

// With profiling on, hands the next kernel launch of this thread an event pair that the runtime
// stamps with the kernel's begin and end.  One launch per scope.
struct ProfScope {
    static hipEvent_t take(moe_ctx *c) {
        hipEvent_t e = nullptr;
        if (!c->free_events.empty()) { e = c->free_events.back(); c->free_events.pop_back(); }
        else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
        return e;
    }
    moe_ctx *ctx; int kernel;
    ProfScope(moe_ctx *c, int k, hipStream_t) : ctx(c), kernel(k) {
        if (!ctx->profiling) return;
        hipEvent_t start = take(ctx), stop = take(ctx);
        if (!start || !stop) return;
        g_launch_timing = LaunchTiming{start, stop};
        ctx->pairs[kernel].push_back(std::make_pair(start, stop));
    }
    ~ProfScope() {
        if (g_launch_timing.stop) {          // nothing was launched inside the scope
            ctx->free_events.push_back(g_launch_timing.start);
            ctx->free_events.push_back(g_launch_timing.stop);
            ctx->pairs[kernel].pop_back();
            g_launch_timing = LaunchTiming{nullptr, nullptr};
        }
    }
};

}  // namespace moespeq

using namespace moespeq;

extern "C" {

int moe_create(moe_ctx **out, int device)
{
    if (!out) return MOE_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return MOE_ERR_HIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return MOE_ERR_HIP;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return MOE_ERR_HIP;   // kernels are gfx950 only
    moe_ctx *c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ERR_HIP;
    c->hip_error[0] = 0;
    c->profiling = false;
    c->device = device;
    c->n_cu = prop.multiProcessorCount;
    c->spin_limit = kDefaultSpinLimit;
    {
        int prev = 0;
        hipError_t e = hipGetDevice(&prev);
        if (e == hipSuccess) e = hipSetDevice(device);
        void *p = nullptr;
        if (e == hipSuccess) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            (void)hipSetDevice(prev);
        }
        if (e != hipSuccess || !p) { delete c; return MOE_ERR_HIP; }
        c->scratch = p;
    }
    strncpy(c->arch, prop.gcnArchName, sizeof(c->arch) - 1);
    *out = c;
    return MOE_OK;
}

int moe_destroy(moe_ctx *ctx)
{
    if (ctx) {
        (void)moe_profile_enable(ctx, 0);
        for (hipEvent_t e : ctx->free_events) (void)hipEventDestroy(e);
    }
    delete ctx;
    return MOE_OK;
}

int moe_profile_enable(moe_ctx *ctx, int enable)
{
    if (!ctx) return MOE_ERR_INVALID_ARG;
    if (!enable) {
        for (auto &v : ctx->pairs) {
            for (auto &p : v) {
                (void)hipEventSynchronize(p.second);
                ctx->free_events.push_back(p.first);
                ctx->free_events.push_back(p.second);
            }
            v.clear();
        }
    }
    ctx->profiling = enable != 0;
    return MOE_OK;
}

int moe_profile_read(moe_ctx *ctx, int kernel, double *total_ms, int64_t *launches)
{
    if (!ctx || kernel < 0 || kernel >= MOE_KERNEL_COUNT || !total_ms || !launches)
        return MOE_ERR_INVALID_ARG;
    double sum = 0.0;
    int64_t n = 0;
    for (auto &p : ctx->pairs[kernel]) {
        hipError_t e = hipEventSynchronize(p.second);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.first, p.second);
        if (e != hipSuccess) return hip_status(ctx, e);
        sum += ms;
        ++n;
        ctx->free_events.push_back(p.first);
        ctx->free_events.push_back(p.second);
    }
    ctx->pairs[kernel].clear();
    *total_ms = sum;
    *launches = n;
    return MOE_OK;
}

const char *moe_kernel_name(int kernel)
{
    static const char *names[MOE_KERNEL_COUNT] = {
        "route_kernel", "plan_kernel", "draft_fused_kernel", "stream_read_kernel",
        "bf16_gateup_kernel", "bf16_down_kernel", "combine_kernel", "union_kernel",
        "prefill_stage_kernel", "prefill_gateup_kernel", "prefill_down_kernel", "prefill_combine_kernel"};
    return (kernel >= 0 && kernel < MOE_KERNEL_COUNT) ? names[kernel] : "";
}

const char *moe_status_string(int status)
{
    switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_WORKSPACE: return "workspace too small or misaligned";
    case MOE_ERR_HIP: return "HIP error";
    case MOE_ERR_MISSING_EXPERT: return "an expert needed by the call is not resident";
    default: return "unknown status";
    }
}

const char *moe_last_hip_error(const moe_ctx *ctx) { return ctx ? ctx->hip_error : ""; }

int moe_validate_desc(const moe_layer_desc *desc) { return check_desc(desc); }

int moe_draft_call_fits(const moe_layer_desc *desc, int T)
{
    if (check_desc(desc) != MOE_OK || check_tokens(desc, T, MOE_MAX_DRAFT_TOKENS) != MOE_OK) return MOE_ERR_INVALID_ARG;
    return draft_fits(make_shape(desc, T), T, false) ? MOE_OK : MOE_ERR_INVALID_ARG;
}

size_t moe_bf16_expert_bytes(const moe_layer_desc *d)
{
    if (check_desc(d) != MOE_OK) return 0;
    return (size_t)3 * d->hidden * d->inter * 2;
}

size_t moe_int4_expert_q_bytes(const moe_layer_desc *d)
{
    if (check_desc(d) != MOE_OK) return 0;
    return (size_t)3 * d->hidden * d->inter / 2;
}

size_t moe_int4_expert_sz_bytes(const moe_layer_desc *d)
{
    if (check_desc(d) != MOE_OK) return 0;
    return (size_t)3 * d->hidden * d->inter / d->group_size * 4;
}

size_t moe_int4_expert_scale_bytes(const moe_layer_desc *d)
{
    if (check_desc(d) != MOE_OK) return 0;
    // two groups (gate/up) and two row tiles (down) share a 16-byte unit
    if ((d->hidden / d->group_size) % 2 || d->hidden % 128) return 0;
    return (size_t)3 * d->hidden * d->inter / d->group_size * 2;
}

int moe_workspace_bytes(const moe_layer_desc *desc, int max_tokens, size_t *bytes)
{
    if (!bytes || check_desc(desc) != MOE_OK) return MOE_ERR_INVALID_ARG;
    if (check_tokens(desc, max_tokens, MOE_MAX_TOKENS) != MOE_OK) return MOE_ERR_INVALID_ARG;
    *bytes = ws_layout(*desc, max_tokens).total;
    return MOE_OK;
}

int moe_workspace_idle_bytes(const moe_layer_desc *desc, size_t *bytes)
{
    if (!bytes || check_desc(desc) != MOE_OK) return MOE_ERR_INVALID_ARG;
    *bytes = ws_layout(*desc, 1).plan;          // counters, status word and router-exchange slots
    return MOE_OK;
}

int moe_workspace_init(moe_ctx *ctx, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx || !workspace || !aligned(workspace, 256) || workspace_bytes < kWsHeadBytes || workspace_bytes % 4)
        return MOE_ERR_INVALID_ARG;
    launch_zero(workspace, workspace_bytes, (hipStream_t)stream);
    return hip_status(ctx, hipGetLastError());
}

int moe_set_draft_spin_limit(moe_ctx *ctx, uint32_t polls)
{
    if (!ctx || polls < 1) return MOE_ERR_INVALID_ARG;
    ctx->spin_limit = polls;
    return MOE_OK;
}

int moe_draft_status(moe_ctx *ctx, const void *workspace, size_t workspace_bytes, int32_t *status, void *stream)
{
    if (!ctx || !workspace || !aligned(workspace, 256) || workspace_bytes < kWsHeadBytes || !status) return MOE_ERR_INVALID_ARG;
    uint32_t word = 0;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(&word, (const char *)workspace + kWsStatusOffset, sizeof word, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_status(ctx, e);
    *status = word == 0 ? MOE_DRAFT_OK : MOE_DRAFT_TIMED_OUT;
    return MOE_OK;
}

int moe_route_topk(moe_ctx *ctx, const moe_layer_desc *desc,
                   const void *x, const void *wr, const float *bias, int T,
                   int32_t *ids, float *w, float *conf,
                   int32_t *counts, int32_t *offsets, int32_t *perm, void *stream)
{
    if (!ctx || check_desc(desc) != MOE_OK || check_tokens(desc, T, MOE_MAX_TOKENS) != MOE_OK)
        return MOE_ERR_INVALID_ARG;
    if (!x || !wr || !ids || !w || !aligned(x, 16) || !aligned(wr, 16) || !aligned(ids, 4) ||
        !aligned(w, 4) || !aligned(conf, 4) || !aligned(bias, 4))
        return MOE_ERR_INVALID_ARG;
    const int nperm = (counts != nullptr) + (offsets != nullptr) + (perm != nullptr);
    if (nperm != 0 && nperm != 3) return MOE_ERR_INVALID_ARG;
    if (!aligned(counts, 4) || !aligned(offsets, 4) || !aligned(perm, 4)) return MOE_ERR_INVALID_ARG;
    const Shape s = make_shape(desc, T);
    hipStream_t st = (hipStream_t)stream;
    { ProfScope p(ctx, MOE_KERNEL_ROUTE, st); launch_route(s, x, wr, bias, ids, w, conf, st); }
    if (nperm) { ProfScope p(ctx, MOE_KERNEL_PLAN, st); launch_perm(s, ids, counts, offsets, perm, st); }
    return hip_status(ctx, hipGetLastError());
}

// Argument checks of a draft call (everything but the workspace)
static int check_draft_args(moe_ctx *ctx, const moe_layer_desc *desc, const void *x, const void *wr,
                            const float *bias, const moe_int4_experts *routed, const void *shared, int T,
                            const float *y, const int32_t *ids_out, const float *conf_out)
{
    if (!ctx || check_desc(desc) != MOE_OK || check_tokens(desc, T, MOE_MAX_DRAFT_TOKENS) != MOE_OK)
        return MOE_ERR_INVALID_ARG;
    if (!x || !wr || !routed || !routed->q || !routed->sz || !y || !ids_out)
        return MOE_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(wr, 16) || !aligned(bias, 4) || !aligned(routed->q, 16) ||
        !aligned(routed->sz, 16) || routed->expert_stride_q % 16 || routed->expert_stride_sz % 16 ||
        !aligned(y, 16) || !aligned(ids_out, 4) || !aligned(conf_out, 4) || !aligned(shared, 16))
        return MOE_ERR_INVALID_ARG;
    const size_t sz_bytes = routed->symmetric ? moe_int4_expert_scale_bytes(desc) : moe_int4_expert_sz_bytes(desc);
    if (sz_bytes == 0 || routed->expert_stride_q < moe_int4_expert_q_bytes(desc) ||
        routed->expert_stride_sz < sz_bytes)
        return MOE_ERR_INVALID_ARG;
    if (desc->n_shared > 0 && !shared) return MOE_ERR_INVALID_ARG;
    if (!draft_fits(make_shape(desc, T), T, routed->symmetric != 0)) return MOE_ERR_INVALID_ARG;     // hidden size too large for T tokens per call
    return MOE_OK;
}

// The launches of a draft call on checked arguments; ws: the call's scratch, laid out by L.
// timed: launches may carry profiling event pairs (which allocates on first use).
static int enqueue_draft(moe_ctx *ctx, const moe_layer_desc *desc, const void *x, const void *wr,
                         const float *bias, const moe_int4_experts *routed, const void *shared, int T,
                         float *y, int32_t *ids_out, float *conf_out, char *ws, const WsLayout &L,
                         hipStream_t st, bool timed)
{
    const Shape s = make_shape(desc, T);
    Plan *plan = (Plan *)(ws + L.plan);
    DraftFusedArgs a;
    memset(&a, 0, sizeof a);
    a.x = x; a.wr = wr; a.bias = bias;
    a.q = routed->q; a.sz = routed->sz;
    a.stride_q = routed->expert_stride_q; a.stride_sz = routed->expert_stride_sz;
    a.symmetric = routed->symmetric ? 1 : 0;
    a.slots = (unsigned long long *)(ws + L.slots);
    a.replica_stride = L.slot_replica_bytes / 8;
    a.tickets = (uint32_t *)(ws + L.tickets);
    a.status = (uint32_t *)(ws + L.tickets + kWsStatusOffset);
    a.spin_limit = ctx->spin_limit;
    a.y = y; a.ids_out = ids_out; a.conf_out = conf_out;
    a.plan = plan; a.shared = shared; a.shared_stride = moe_bf16_expert_bytes(desc);
    // the workgroups that reduce the router rows (the first min(E, grid) of the launch) must be
    // running while the others wait for them
    if (!draft_producers_resident(s, a, ctx->n_cu)) return MOE_ERR_INVALID_ARG;
    if (!timed) {
        launch_draft_fused(s, a, ctx->n_cu, st);
        if (s.S > 0) {
            launch_bf16_gateup(s, plan, 0, s.S, x, ws + L.hb, ws + L.hb_lo, st);
            launch_bf16_down_add(s, plan, 0, s.S, ws + L.hb, ws + L.hb_lo, y, st);
        }
        return hip_status(ctx, hipGetLastError());
    }
    { ProfScope p(ctx, MOE_KERNEL_DRAFT_FUSED, st); launch_draft_fused(s, a, ctx->n_cu, st); }
    if (s.S > 0) {   // shared experts stay 16-bit in the draft model (section 3.4.2)
        { ProfScope p(ctx, MOE_KERNEL_BF16_GATEUP, st);
          launch_bf16_gateup(s, plan, 0, s.S, x, ws + L.hb, ws + L.hb_lo, st); }
        // the down kernel adds the shared experts' outputs to y itself (fp32 atomics on top of
        // the routed experts' sum): no combine launch
        { ProfScope p(ctx, MOE_KERNEL_BF16_DOWN, st);
          launch_bf16_down_add(s, plan, 0, s.S, ws + L.hb, ws + L.hb_lo, y, st); }
    }
    return hip_status(ctx, hipGetLastError());
}

int moe_draft_layer_int4(moe_ctx *ctx, const moe_layer_desc *desc,
                         const void *x, const void *wr, const float *bias,
                         const moe_int4_experts *routed, const void *shared, int T,
                         float *y, int32_t *ids_out, float *conf_out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = check_draft_args(ctx, desc, x, wr, bias, routed, shared, T, y, ids_out, conf_out);
    if (rc != MOE_OK) return rc;
    const WsLayout L = ws_layout(*desc, T);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    return enqueue_draft(ctx, desc, x, wr, bias, routed, shared, T, y, ids_out, conf_out, (char *)workspace, L,
                         (hipStream_t)stream, true);
}

size_t moe_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int moe_draft_layer_int4_noalloc(moe_ctx *ctx, const moe_layer_desc *desc,
                                 const void *x, const void *wr, const float *bias,
                                 const moe_int4_experts *routed, const void *shared, int T,
                                 float *y, int32_t *ids_out, float *conf_out, void *stream)
{
    const int rc = check_draft_args(ctx, desc, x, wr, bias, routed, shared, T, y, ids_out, conf_out);
    if (rc != MOE_OK) return rc;
    const WsLayout L = ws_layout(*desc, T);
    if (L.total > kStaticScratchBytes) return MOE_ERR_WORKSPACE;     // shape beyond the static scratch array
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device) return MOE_ERR_INVALID_ARG;   // ctx->scratch is this device's copy
    char *ws = (char *)ctx->scratch;         // the device address from hipGetSymbolAddress, never the array's name
    hipStream_t st = (hipStream_t)stream;
    // The array keeps whatever the last call on this GPU left.  The part that must start at zero
    // (ticket counters and exchange slots) is cleared by a fill kernel, which is also safe
    // under stream capture.
    launch_zero(ws + L.tickets, L.plan - L.tickets, st);
    return enqueue_draft(ctx, desc, x, wr, bias, routed, shared, T, y, ids_out, conf_out, ws, L, st, false);
}

// workspace of a prefill call: routing weights, sorted assignment indices and slots [T k], the
// item count (one 256-byte line), the items, the operand tiles of x and of h (two planes) with
// their tile row sums, and the per-slot outputs.
// With shared experts: two plans (full chunk, ragged last chunk) and the buffers of one chunk of
// `chunk` tokens through the bf16 kernels.
struct PrefillLayout {
    size_t w_all, sorted, slot_of, n_items, items, xt, x_sums, h_hi, h_lo, h_sums, obuf,
        plan_full, plan_tail, shared_ws, total;
    int max_items, chunk;
};
static PrefillLayout prefill_layout(const moe_layer_desc &d, int T)
{
    PrefillLayout L;
    const size_t n = (size_t)T * d.top_k;
    // sum over experts of ceil(count / chunk) <= n / chunk + number of experts that occur
    L.max_items = (int)(n / kPrefillChunk + ((size_t)d.n_experts < n ? (size_t)d.n_experts : n));
    const PrefillBuffers B = prefill_buffers(d, L.max_items);
    size_t o = 0;
    L.w_all = o;   o += align256(n * 4);
    L.sorted = o;  o += align256(n * 4);
    L.slot_of = o; o += align256(n * 4);
    L.n_items = o; o += 256;
    L.items = o;   o += align256((size_t)L.max_items * sizeof(PrefillItem));
    L.xt = o;      o += align256(B.xt);
    L.x_sums = o;  o += align256(B.x_sums);
    L.h_hi = o;    o += align256(B.h_plane);
    L.h_lo = o;    o += align256(B.h_plane);
    L.h_sums = o;  o += align256(B.h_sums);
    L.obuf = o;    o += align256(B.obuf);
    L.chunk = MOE_MAX_ASSIGN / d.top_k < MOE_MAX_TOKENS ? MOE_MAX_ASSIGN / d.top_k : MOE_MAX_TOKENS;
    L.plan_full = L.plan_tail = L.shared_ws = o;
    if (d.n_shared > 0) {
        L.plan_full = o; o += align256(sizeof(Plan));
        L.plan_tail = o; o += align256(sizeof(Plan));
        L.shared_ws = o; o += ws_layout(d, L.chunk).total;
    }
    L.total = o;
    return L;
}

static int check_prefill(const moe_layer_desc *d, int T)
{
    if (check_desc(d) != MOE_OK) return MOE_ERR_INVALID_ARG;
    if (T < 1 || T > MOE_MAX_PREFILL_TOKENS) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

int moe_prefill_workspace_bytes(const moe_layer_desc *desc, int T, size_t *bytes)
{
    if (!bytes || check_prefill(desc, T) != MOE_OK) return MOE_ERR_INVALID_ARG;
    *bytes = prefill_layout(*desc, T).total;
    return MOE_OK;
}

int moe_draft_prefill_int4(moe_ctx *ctx, const moe_layer_desc *desc,
                           const void *x, const void *wr, const float *bias,
                           const moe_int4_experts *routed, const void *shared, int T,
                           float *y, int32_t *ids_out, float *conf_out,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx || check_prefill(desc, T) != MOE_OK) return MOE_ERR_INVALID_ARG;
    if (!x || !wr || !routed || !routed->q || !routed->sz || !y || !ids_out)
        return MOE_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(wr, 16) || !aligned(bias, 4) || !aligned(routed->q, 16) ||
        !aligned(routed->sz, 16) || routed->expert_stride_q % 16 || routed->expert_stride_sz % 16 ||
        !aligned(y, 16) || !aligned(ids_out, 4) || !aligned(conf_out, 4) || !aligned(shared, 16))
        return MOE_ERR_INVALID_ARG;
    if (desc->n_shared > 0 && !shared) return MOE_ERR_INVALID_ARG;
    const size_t sz_bytes = routed->symmetric ? moe_int4_expert_scale_bytes(desc) : moe_int4_expert_sz_bytes(desc);
    if (sz_bytes == 0 || routed->expert_stride_q < moe_int4_expert_q_bytes(desc) ||
        routed->expert_stride_sz < sz_bytes)
        return MOE_ERR_INVALID_ARG;
    const Shape s = make_shape(desc, T);
    const PrefillLayout L = prefill_layout(*desc, T);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return MOE_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    PrefillCall p;
    p.x = x; p.q = routed->q; p.sz = routed->sz;
    p.stride_q = routed->expert_stride_q; p.stride_sz = routed->expert_stride_sz;
    p.symmetric = routed->symmetric ? 1 : 0;
    p.items = (const PrefillItem *)(ws + L.items); p.n_items = (const int32_t *)(ws + L.n_items);
    p.sorted = (const int32_t *)(ws + L.sorted); p.slot_of = (const int32_t *)(ws + L.slot_of);
    p.w_all = (const float *)(ws + L.w_all);
    p.xt = ws + L.xt; p.x_sums = (float *)(ws + L.x_sums);
    p.h_hi = ws + L.h_hi; p.h_lo = ws + L.h_lo; p.h_sums = (float *)(ws + L.h_sums);
    p.obuf = (float *)(ws + L.obuf);
    p.y = y;
    { ProfScope t(ctx, MOE_KERNEL_ROUTE, st); launch_route(s, x, wr, bias, ids_out, (float *)(ws + L.w_all), conf_out, st); }
    { ProfScope t(ctx, MOE_KERNEL_PLAN, st);
      launch_prefill_plan(ids_out, T * s.k, s.E, (int32_t *)(ws + L.sorted), (int32_t *)(ws + L.slot_of),
                          (PrefillItem *)(ws + L.items), (int32_t *)(ws + L.n_items), st); }
    { ProfScope t(ctx, MOE_KERNEL_PREFILL_STAGE, st); launch_prefill_stage(s, p, L.max_items, st); }
    { ProfScope t(ctx, MOE_KERNEL_PREFILL_GATEUP, st); launch_prefill_gateup(s, p, L.max_items, st); }
    { ProfScope t(ctx, MOE_KERNEL_PREFILL_DOWN, st); launch_prefill_down(s, p, L.max_items, st); }
    { ProfScope t(ctx, MOE_KERNEL_PREFILL_COMBINE, st); launch_prefill_combine(s, p, st); }
    if (s.S > 0) {
        // shared experts stay 16-bit (section 3.4.2): chunks of tokens through the bf16 kernels,
        // added to y; the intermediate keeps a bf16 remainder as in the draft call
        const size_t bf16_bytes = moe_bf16_expert_bytes(desc);
        const WsLayout W = ws_layout(*desc, L.chunk);
        char *sw = ws + L.shared_ws;
        Shape sc = s;
        sc.T = L.chunk;
        Plan *full = (Plan *)(ws + L.plan_full), *tail = (Plan *)(ws + L.plan_tail);
        if (T >= L.chunk) launch_shared_plan(sc, full, shared, bf16_bytes, st);
        for (int t0 = 0; t0 < T; t0 += L.chunk) {
            const int tc = T - t0 < L.chunk ? T - t0 : L.chunk;
            sc.T = tc;
            Plan *plan = full;
            if (tc < L.chunk) { plan = tail; launch_shared_plan(sc, tail, shared, bf16_bytes, st); }
            const char *xc = (const char *)x + (size_t)t0 * s.H * 2;
            { ProfScope p(ctx, MOE_KERNEL_BF16_GATEUP, st);
              launch_bf16_gateup(sc, plan, 0, s.S, xc, sw + W.hb, sw + W.hb_lo, st); }
            { ProfScope p(ctx, MOE_KERNEL_BF16_DOWN, st);
              launch_bf16_down(sc, plan, 0, s.S, sw + W.hb, sw + W.hb_lo, (float *)(sw + W.obuf), st); }
            { ProfScope p(ctx, MOE_KERNEL_COMBINE, st);
              launch_combine(sc, plan, nullptr, 0, (const float *)(sw + W.obuf), 1, 0, y + (size_t)t0 * s.H, st); }
        }
    }
    return hip_status(ctx, hipGetLastError());
}

int moe_expert_union(moe_ctx *ctx, const int32_t *ids, int n_ids, int n_experts,
                     const int32_t *slot_of_expert, uint64_t *mask, int32_t *list, int32_t *n_list,
                     int32_t *missing, int32_t *n_missing, void *stream)
{
    if (!ctx || n_ids < 0 || n_experts < 1 || n_experts > MOE_MAX_EXPERTS) return MOE_ERR_INVALID_ARG;
    if ((n_ids > 0 && !ids) || !mask || !list || !n_list || !n_missing) return MOE_ERR_INVALID_ARG;
    if (slot_of_expert && !missing) return MOE_ERR_INVALID_ARG;
    if (!aligned(ids, 4) || !aligned(slot_of_expert, 4) || !aligned(mask, 8) || !aligned(list, 4) ||
        !aligned(n_list, 4) || !aligned(missing, 4) || !aligned(n_missing, 4))
        return MOE_ERR_INVALID_ARG;
    { ProfScope p(ctx, MOE_KERNEL_UNION, (hipStream_t)stream);
      launch_union(ids, n_ids, n_experts, slot_of_expert, mask, list, n_list, missing, n_missing,
                   (hipStream_t)stream); }
    return hip_status(ctx, hipGetLastError());
}

int moe_verify_layer_bf16(moe_ctx *ctx, const moe_layer_desc *desc,
                          const void *x, const void *wr, const float *bias,
                          const void *slot_pool, size_t slot_stride, const int32_t *slot_of_expert,
                          const void *shared, int T, int flags,
                          void *y, int32_t *ids_out, int32_t *missing, int32_t *n_missing,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx || check_desc(desc) != MOE_OK || check_tokens(desc, T, MOE_MAX_TOKENS) != MOE_OK)
        return MOE_ERR_INVALID_ARG;
    if (flags & ~(MOE_VERIFY_ACCUMULATE | MOE_VERIFY_ONLY_LISTED | MOE_VERIFY_STRICT))
        return MOE_ERR_INVALID_ARG;
    if (!x || !wr || !slot_pool || !slot_of_expert || !y || !missing || !n_missing)
        return MOE_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(wr, 16) || !aligned(bias, 4) || !aligned(slot_pool, 16) ||
        slot_stride % 16 || slot_stride < moe_bf16_expert_bytes(desc) || !aligned(slot_of_expert, 4) ||
        !aligned(shared, 16) || !aligned(y, 8) || !aligned(ids_out, 4) || !aligned(missing, 4) ||
        !aligned(n_missing, 4))
        return MOE_ERR_INVALID_ARG;
    if (desc->n_shared > 0 && !shared) return MOE_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(*desc, T);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return MOE_ERR_WORKSPACE;

    const Shape s = make_shape(desc, T);
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    Plan *plan = (Plan *)(ws + L.plan);
    PlanArgs a;
    memset(&a, 0, sizeof a);
    a.plan = plan; a.mode = 1;
    a.w0 = slot_pool; a.stride0 = slot_stride;
    a.slot_of_expert = slot_of_expert;
    a.shared = shared; a.shared_stride = moe_bf16_expert_bytes(desc);
    a.flags = flags;
    a.ids_out = ids_out;
    a.missing = missing; a.n_missing = n_missing;
    // router and plan in one launch; its arrival counter sits behind the draft kernel's tickets
    { ProfScope p(ctx, MOE_KERNEL_ROUTE, st);
      launch_route_plan(s, x, wr, bias, a, (double *)(ws + L.vlogits),
                        (uint32_t *)(ws + L.tickets + kWsTokenArrivalsOffset),
                        (uint32_t *)(ws + L.tickets + kWsArrivalsOffset), st); }
    const int nexp = s.S + (s.E < s.T * s.k ? s.E : s.T * s.k);
    { ProfScope p(ctx, MOE_KERNEL_BF16_GATEUP, st); launch_bf16_gateup(s, plan, 0, nexp, x, ws + L.hb, nullptr, st); }
    { ProfScope p(ctx, MOE_KERNEL_BF16_DOWN, st);
      launch_bf16_down(s, plan, 0, nexp, ws + L.hb, nullptr, (float *)(ws + L.obuf), st); }
    { ProfScope p(ctx, MOE_KERNEL_COMBINE, st);
      launch_combine(s, plan, (const float *)(ws + L.obuf), 1, (const float *)(ws + L.obuf),
                     (flags & MOE_VERIFY_ACCUMULATE) ? 1 : 0, 1, y, st); }
    int rc = hip_status(ctx, hipGetLastError());
    if (rc != MOE_OK) return rc;
    if (flags & MOE_VERIFY_STRICT) {
        int32_t nm = 0;
        hipError_t e = hipMemcpyAsync(&nm, n_missing, sizeof nm, hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return hip_status(ctx, e);
        if (nm != 0) return MOE_ERR_MISSING_EXPERT;
    }
    return MOE_OK;
}

int moe_expert_copy_async(moe_ctx *ctx, void *dst, const void *src, size_t bytes,
                          void *copy_stream, void *done_event)
{
    if (!ctx || !dst || !src || bytes == 0) return MOE_ERR_INVALID_ARG;
    hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, (hipStream_t)copy_stream);
    if (e == hipSuccess && done_event) e = hipEventRecord((hipEvent_t)done_event, (hipStream_t)copy_stream);
    return hip_status(ctx, e);
}

int moe_stream_read_probe(moe_ctx *ctx, const void *src, size_t bytes, int workgroups, void *sink,
                          void *stream)
{
    if (!ctx || !src || !sink || bytes < 1024 || bytes % 1024 || ((uintptr_t)src & 15) ||
        ((uintptr_t)sink & 3) || workgroups < 1 || workgroups > 65536)
        return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    { ProfScope p(ctx, MOE_KERNEL_STREAM_READ, st); launch_stream_read(src, bytes, workgroups, sink, st); }
    return hip_status(ctx, hipGetLastError());
}

}  // extern "C"
