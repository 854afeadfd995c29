// Internal: the per-call execution plan that the route/plan kernels leave in the workspace
// and that the expert kernels read, plus the host-side launcher prototypes of each .hip file.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "../../include/moespeq.h"

namespace moespeq {

// Every kernel of the library is launched through launch().  When a timing pair is pending on
// this host thread (set by the profiling mode of the C ABI) the launch carries it: the runtime
// then stamps `start` / `stop` with the begin and end of the kernel's own execution, which is the
// duration a kernel trace reports, without the gaps an event recorded before and after would add.
struct LaunchTiming { hipEvent_t start, stop; };
extern thread_local LaunchTiming g_launch_timing;

template <typename K, typename... A>
inline void launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, A... args)
{
    if (g_launch_timing.stop) {
        const LaunchTiming t = g_launch_timing;
        g_launch_timing = LaunchTiming{nullptr, nullptr};
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, t.start, t.stop, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
    }
}

constexpr int kMaxRows = MOE_MAX_ASSIGN + MOE_MAX_TOKENS * MOE_MAX_SHARED;   // routed + shared rows
constexpr int kMaxActive = MOE_MAX_ASSIGN + MOE_MAX_SHARED;                   // distinct experts per call

// A "row" is one (token, expert) pair the expert kernels work on.  Rows of one expert are
// contiguous: routed rows are the stable permutation of the assignments (section 3.4.4),
// shared-expert rows follow, one per token and shared expert.
struct Plan {
    int32_t n_active;                 // experts the expert kernels run (routed present + shared)
    int32_t n_routed_active;
    int32_t n_rows;                   // T*k + T*S
    int32_t n_missing;
    int32_t ids[MOE_MAX_ASSIGN];      // [T,k]
    float   w[MOE_MAX_ASSIGN];
    float   conf[MOE_MAX_ASSIGN];
    int32_t count[MOE_MAX_EXPERTS];
    int32_t off[MOE_MAX_EXPERTS + 1];
    int32_t perm[MOE_MAX_ASSIGN];
    int32_t act_expert[kMaxActive];   // expert id (>= E: shared expert id - E)
    int32_t act_off[kMaxActive];      // first row
    int32_t act_cnt[kMaxActive];      // number of rows (tokens of that expert)
    uint64_t act_w0[kMaxActive];      // weights: bf16 blob / int4 codes blob
    uint64_t act_w1[kMaxActive];      // int4 scale-zero blob
    int32_t row_tok[kMaxRows];        // token of a row
    float   row_w[kMaxRows];          // routing weight of a row (1 for shared)
    int32_t row_live[kMaxRows];       // 0: expert absent, the row's output must be skipped
};

struct Shape {
    int T, H, E, I, k, S, g, renorm;
};

// Workspace carve-up (byte offsets from a 256-byte aligned base).  [tickets, plan) must be
// zero between calls ("idle state"): moe_workspace_init establishes it, the draft kernel
// restores it.  Their sizes do not depend on T, so the idle region is the same for every call.
constexpr int kDraftSlotReplicas = 16;   // copies of the draft kernel's router-exchange slots
// inside the first block (the `tickets` block, kWsHeadBytes): the verify call's arrival counter and the
// draft calls' status word (0: fine, 1: a wait for the router result ran out of polls)
constexpr size_t kWsArrivalsOffset = 128, kWsStatusOffset = 192;
constexpr size_t kWsTokenArrivalsOffset = 256;           // MOE_MAX_TOKENS counters of the verify call's router
constexpr size_t kWsHeadBytes = 512;                     // size of that first block
constexpr uint32_t kDefaultSpinLimit = 1u << 22;

struct WsLayout {
    // tickets: one counter; slots: [MOE_MAX_DRAFT_TOKENS, E] x {fp64 logit, 64-bit tag} of the
    // draft kernel's router exchange; hb / hb_lo: bf16 intermediate and its bf16 remainder;
    // obuf: fp32 [rows,H] expert outputs
    size_t tickets, slots, slot_replica_bytes, plan, vlogits, hb, hb_lo, obuf, total;
};
WsLayout ws_layout(const moe_layer_desc &d, int max_tokens);

// route.hip
void launch_route(const Shape &s, const void *x, const void *wr, const float *bias,
                  int32_t *ids, float *w, float *conf, hipStream_t st);
void launch_perm(const Shape &s, const int32_t *ids, int32_t *count, int32_t *off,
                 int32_t *perm, hipStream_t st);
struct PlanArgs {
    Plan *plan;
    int mode;                          // 0 draft (int4 routed, all present), 1 verify (slot table)
    const void *w0; size_t stride0;    // draft: codes base / stride; verify: slot pool / stride
    const void *w1; size_t stride1;    // draft: scale-zero base / stride
    const int32_t *slot_of_expert;
    const void *shared; size_t shared_stride;
    int flags;
    int32_t *ids_out; float *conf_out;
    int32_t *missing; int32_t *n_missing;
};
void launch_plan(const Shape &s, const PlanArgs &a, hipStream_t st);
// router + plan in one launch; logits: [T, E] fp64 scratch; token_arrivals [MOE_MAX_TOKENS] and
// arrivals: counters in the workspace, zero between launches
void launch_route_plan(const Shape &s, const void *x, const void *wr, const float *bias, const PlanArgs &a,
                       double *logits, uint32_t *token_arrivals, uint32_t *arrivals, hipStream_t st);
// plan of the S shared experts alone over s.T tokens
void launch_shared_plan(const Shape &s, Plan *plan, const void *shared, size_t shared_stride, hipStream_t st);
void launch_union(const int32_t *ids, int n_ids, int E, const int32_t *slot,
                  uint64_t *mask, int32_t *list, int32_t *n_list,
                  int32_t *missing, int32_t *n_missing, hipStream_t st);

// Work item of the draft call over a long run of tokens: up to kPrefillChunk assignments of one
// expert, sorted[first .. first + cnt).  Item i owns slots [64 i, 64 i + cnt).
constexpr int kPrefillChunk = 64;
struct PrefillItem { int32_t expert, first, cnt, pad; };

// draft_int4.hip (a call of 2 to 8 tokens) and draft_slice.hip (a call of one token)
struct DraftFusedArgs {
    const void *x, *wr; const float *bias;
    const void *q, *sz; size_t stride_q, stride_sz;
    int symmetric;                     // sz holds scale blobs (z = 8)
    unsigned long long *slots; size_t replica_stride; uint32_t *tickets;
    uint32_t *status; uint32_t spin_limit;
    float *y; int32_t *ids_out; float *conf_out;
    Plan *plan; const void *shared; size_t shared_stride;
};
// n_cu: compute units of the device (the launch is persistent, at most one workgroup per unit)
void launch_draft_fused(const Shape &s, const DraftFusedArgs &a, int n_cu, hipStream_t st);
// whether the x copy and the entry buffers of a call with `tokens` tokens (1-8) fit into LDS
bool draft_fits(const Shape &s, int tokens, bool symmetric);
// whether the workgroups of the call's launch that reduce the router rows are all resident at once
// (occupancy of the kernel the call will run x compute units)
bool draft_producers_resident(const Shape &s, const DraftFusedArgs &a, int n_cu);
// draft_slice.hip: the call with ONE token (router inside the launch), one workgroup per
// (expert, slice) work item
void launch_draft_one_token(const Shape &s, const DraftFusedArgs &a, hipStream_t st);
bool draft_one_token_fits(const Shape &s);
int draft_one_token_resident(const Shape &s, const DraftFusedArgs &a, int n_cu);   // workgroups resident at once
void launch_zero(void *p, size_t bytes, hipStream_t st);
void launch_stream_read(const void *src, size_t bytes, int workgroups, void *sink, hipStream_t st);

// draft_prefill.hip: a routed run of tokens.  Byte sizes of the buffers a call with at most
// max_items work items needs (h_plane: each of the two planes of h), then the launches in order.
struct PrefillBuffers { size_t xt, x_sums, h_plane, h_sums, obuf; };
PrefillBuffers prefill_buffers(const moe_layer_desc &d, int max_items);
struct PrefillCall {
    const void *x;                     // [T,H] bf16
    const void *q, *sz; size_t stride_q, stride_sz; int symmetric;
    const PrefillItem *items; const int32_t *n_items; const int32_t *sorted; const int32_t *slot_of;
    const float *w_all;                // routing weight of every assignment [T k]
    void *xt; float *x_sums; void *h_hi, *h_lo; float *h_sums; float *obuf;
    float *y;                          // [T,H] fp32, written (not accumulated)
};
void launch_prefill_plan(const int32_t *ids, int n, int E, int32_t *sorted, int32_t *slot_of,
                         PrefillItem *items, int32_t *n_items, hipStream_t st);
void launch_prefill_stage(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st);
void launch_prefill_gateup(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st);
void launch_prefill_down(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st);
void launch_prefill_combine(const Shape &s, const PrefillCall &p, hipStream_t st);

// expert_bf16.hip
// hb_lo != nullptr: the intermediate is kept as a bf16 hi + lo pair (draft-pass precision)
void launch_bf16_gateup(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                        const void *x, void *hb, void *hb_lo, hipStream_t st);
void launch_bf16_down(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                      const void *hb, const void *hb_lo, float *obuf, hipStream_t st);
// the same product, each row's outputs added to y[row_tok[row]] (fp32, [T,H]) with atomics; the
// intermediate is the bf16 hi + lo pair
void launch_bf16_down_add(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                          const void *hb, const void *hb_lo, float *y, hipStream_t st);
// y[t] = (accumulate ? y[t] : 0) + sum over the token's live routed rows of
// sum_{split < nsplit} routed[split][row] + sum over its live shared rows of obuf[row];
// routed is [nsplit][T*k][H] fp32, obuf is [rows][H] fp32 indexed by row number.
void launch_combine(const Shape &s, const Plan *plan, const float *routed, int nsplit,
                    const float *obuf, int accumulate, int out_bf16, void *y, hipStream_t st);

}  // namespace moespeq
