/*
 * moespeq.h -- C ABI of the MI355X (gfx950) MoE-layer library for MoE-SpeQ-style speculative
 * quantized decoding (arXiv 2511.14102).
 *
 * The library runs the Mixture-of-Experts layer forward of the paper's execution engine
 * (section 3.4): once per draft step on group-wise int4 expert weights, emitting the
 * expert-id sets that fill the Expert Lookahead Buffer (section 3.3.1), and once per verify
 * step in bf16 over the K+1 speculative tokens against experts held in a VRAM expert cache
 * that is addressed through a slot table (sections 3.3.2, 3.4.4).
 *
 * General rules
 *  - Plain C linkage, plain pointers and sizes.  Unless a parameter says "host", every data
 *    pointer is a DEVICE pointer owned by the caller; the library keeps no pointer after a
 *    call returns and allocates nothing per call (section 4.1.2: no run-time allocation in
 *    the hot path).  `stream` parameters are hipStream_t handles passed as void* (NULL = the
 *    default stream); events are hipEvent_t handles passed as void*.
 *  - Every call validates its arguments on the host, enqueues its kernels on `stream` and
 *    returns; outputs are valid once the stream has reached that point.  No call
 *    synchronises, except moe_verify_layer_bf16 with MOE_VERIFY_STRICT.
 *  - Return value: MOE_OK or a negative status.  On MOE_ERR_INVALID_ARG / MOE_ERR_WORKSPACE
 *    nothing has been enqueued.  After MOE_ERR_HIP, moe_last_hip_error() names the HIP error.
 *  - Inputs must be finite; NaN / Inf activations or weights give unspecified outputs.
 *  - One moe_ctx may be used from one host thread at a time.  Calls that share a workspace
 *    must be ordered on one stream (or by events).
 *
 * Shapes: T tokens, H hidden, E routed experts, I intermediate (SwiGLU), k top-k, g int4 group
 * size, S shared experts.  Assignment index a = t * k + j (token-major, j = rank).
 * Limits: 1 <= T <= MOE_MAX_TOKENS (draft: MOE_MAX_DRAFT_TOKENS), E <= MOE_MAX_EXPERTS,
 * k <= min(E, MOE_MAX_TOPK), T * k <= MOE_MAX_ASSIGN, S <= MOE_MAX_SHARED, H and I multiples
 * of 64, g in {32, 64, 128} dividing both H and I.  What a draft call keeps in LDS must stay under
 * 140 KiB, else MOE_ERR_INVALID_ARG (moe_draft_call_fits tells).  One token: 2 H + 16 + 4 H / g bytes
 * (its copy and group sums), plus 12 E + 8 bytes of routing scratch when E > 32 (H <= 65536).  Two to
 * eight tokens, T rounded up to 2, 4 or 8: T (2 H + 16 + 4 H / g) + 12 T E bytes (rounded up to 16) plus
 * 16 KiB x (ceil(ceil(H / g / 8) / 4) + ceil(ceil(H / 64 / 8) / 4)) for the scale / zero entries of one
 * work item (in the symmetric format H / g and H / 64 count pairs).  The prefill call keeps a fixed
 * 34 KiB whatever the shape.
 *
 * Kernel-native weight layouts (part of the ABI; pack.py builds them from row-major arrays)
 *
 *  bf16 matrix W[R][C] (R outputs, C inputs; R % 16 == 0, C % 32 == 0), "tile16x32":
 *      a sequence of 1 KiB tiles, tile index (R/16-major) tile = (r / 16) * (C / 32) + c / 32;
 *      inside a tile 64 lanes x 8 bf16:  lane = ((c % 32) / 8) * 16 + r % 16,  element c % 8.
 *      (This is the A-operand register image of the 16x16x32 bf16 MFMA, so one 16-byte load
 *      per lane fetches one tile.)
 *  bf16 expert blob = [gate I x H | up I x H | down H x I], each tile16x32, contiguous,
 *      moe_bf16_expert_bytes() bytes.  One blob fills one slot of the expert cache.
 *
 *  int4 expert: codes q in 0..15, fp16 scale s and zero z per (row, group of g consecutive
 *  inputs), W = (q - z) * s.  8 codes of one row (input columns 8j .. 8j + 7) are one
 *  little-endian 32-bit word; code number n of the word sits in bits [4p, 4p + 4) with
 *  p = n / 2 for even n and p = 4 + n / 2 for odd n (so `(word >> 4i) & 0x000F000F` is the pair
 *  of codes 2i, 2i + 1).  Words are grouped in 1 KiB tiles of 64 lanes x 4 words in the register
 *  image of a 16x16x32 MFMA operand: lane = chunk * 16 + r holds, for row block d = 0..3 (word d),
 *  the word of row (d, r) and input chunk `chunk` (8 columns) of the tile's 32 columns.
 *    gate/up part ("slices" of 32 intermediate rows, I / 32 of them): tile (slice, u) for input
 *      unit u = c / 32 at index slice * (H / 32) + u; row (d, r) is gate row 32 slice + 16 d + r
 *      for d < 2 and up row 32 slice + 16 (d - 2) + r for d >= 2.
 *    down part, after the (I / 32) * (H / 32) gate/up tiles: tile (slice, rt) at index
 *      slice * (H / 64) + rt; row (d, r) is output row 64 rt + 16 d + r, the 32 columns are
 *      input columns [32 slice, 32 slice + 32).
 *    codes blob = moe_int4_expert_q_bytes() = 3 H I / 2 bytes.
 *  scale/zero blob: 4-byte entries (fp16 s in the low half, fp16 z in the high half), four
 *  consecutive entries d = 0..3 for each r:
 *    gate/up part: entry ((slice * (H / g) + group) * 16 + r) * 4 + d, rows (d, r) as above;
 *    down part, after the (I / 32) * (H / g) * 64 gate/up entries: entry
 *      ((group * (H / 64) + rt) * 16 + r) * 4 + d, group = input column / g.
 *    moe_int4_expert_sz_bytes() = 3 H I / g * 4 bytes.
 *  scale blob of the symmetric format (z = 8 for every group, the usual signed 4-bit weight
 *  q - 8; moe_int4_experts.symmetric != 0): 2-byte entries (fp16 s), no zeros.  Two groups
 *  (gate/up) or two row tiles (down) share one 16-byte unit per r, which holds the four
 *  entries d = 0..3 of the even one and then those of the odd one:
 *    gate/up part: entry (((slice * (H / g / 2) + group / 2) * 16 + r) * 2 + group % 2) * 4 + d;
 *    down part, after the (I / 32) * (H / g) * 64 gate/up entries: entry
 *      ((((group * (H / 128)) + rt / 2) * 16 + r) * 2 + rt % 2) * 4 + d.
 *    moe_int4_expert_scale_bytes() = 3 H I / g * 2 bytes.  Needs H / g even and H % 128 == 0.
 */
#ifndef MOESPEQ_H
#define MOESPEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_TOKENS        16
#define MOE_MAX_DRAFT_TOKENS  8
#define MOE_MAX_PREFILL_TOKENS 4096
#define MOE_MAX_EXPERTS       256
#define MOE_MAX_TOPK          16
#define MOE_MAX_ASSIGN        128
#define MOE_MAX_SHARED        4

#define MOE_OK                   0
#define MOE_ERR_INVALID_ARG     (-1)
#define MOE_ERR_WORKSPACE       (-2)
#define MOE_ERR_HIP             (-3)
#define MOE_ERR_MISSING_EXPERT  (-4)

/* flags of moe_verify_layer_bf16 */
#define MOE_VERIFY_ACCUMULATE   1   /* y += result instead of y = result                    */
#define MOE_VERIFY_ONLY_LISTED  2   /* only experts listed in `missing` on entry; no shared */
#define MOE_VERIFY_STRICT       4   /* synchronise; MOE_ERR_MISSING_EXPERT if any is absent */

typedef struct moe_ctx moe_ctx;      /* opaque: device number and properties, no weights */

typedef struct moe_layer_desc {
    int32_t hidden;        /* H */
    int32_t n_experts;     /* E routed experts */
    int32_t inter;         /* I */
    int32_t top_k;         /* k */
    int32_t n_shared;      /* S always-on shared experts (bf16 in both passes) */
    int32_t group_size;    /* g in {32, 64, 128} (used by the draft calls; every call validates it) */
    int32_t renormalize;   /* nonzero: routing weights divided by their sum over the k */
} moe_layer_desc;

/* Routed experts of the draft model: expert e's codes at q + e * expert_stride_q, its
 * scale/zero blob at sz + e * expert_stride_sz (device pointers, 16-byte aligned strides). */
typedef struct moe_int4_experts {
    const void *q;
    const void *sz;
    size_t expert_stride_q;
    size_t expert_stride_sz;
    int32_t symmetric;     /* nonzero: sz holds scale blobs of the symmetric format, z = 8 */
} moe_int4_experts;

/* ---- context and helpers (host only) ------------------------------------------------- */

/* Creates a context for HIP device `device` (checks that it is a gfx950 part).
 * Errors: MOE_ERR_INVALID_ARG (out == NULL), MOE_ERR_HIP (no such device / not gfx950). */
int moe_create(moe_ctx **out, int device);
int moe_destroy(moe_ctx *ctx);

/* Static, never NULL. */
const char *moe_status_string(int status);
/* Name of the last HIP error seen by `ctx` ("" if none); valid until the next call on ctx. */
const char *moe_last_hip_error(const moe_ctx *ctx);

/* MOE_OK if `desc` is a shape the kernels support (the limits above), else
 * MOE_ERR_INVALID_ARG.  Needs no device. */
int moe_validate_desc(const moe_layer_desc *desc);

/* MOE_OK if a draft call with T tokens (1 .. MOE_MAX_DRAFT_TOKENS; the prefill call always fits)
 * fits the LDS limit stated above for this shape, else MOE_ERR_INVALID_ARG.  Needs no device. */
int moe_draft_call_fits(const moe_layer_desc *desc, int T);

/* Sizes of the packed weight blobs of one expert (0 if desc is invalid). */
size_t moe_bf16_expert_bytes(const moe_layer_desc *desc);
size_t moe_int4_expert_q_bytes(const moe_layer_desc *desc);
size_t moe_int4_expert_sz_bytes(const moe_layer_desc *desc);
/* scale blob of the symmetric format; 0 also when the shape does not allow that format */
size_t moe_int4_expert_scale_bytes(const moe_layer_desc *desc);

/* Bytes of device workspace that moe_draft_layer_int4 / moe_verify_layer_bf16 need for up to
 * `max_tokens` tokens per call (256-byte aligned base). */
int moe_workspace_bytes(const moe_layer_desc *desc, int max_tokens, size_t *bytes);

/* Puts a workspace into its idle state (enqueues a fill kernel on `stream`; workspace_bytes a
 * multiple of 4).  Required once after allocation, before the first moe_draft_layer_int4 OR
 * moe_verify_layer_bf16 call on it, and again after a draft call that timed out (below).  The first
 * 512 bytes and the slot area behind them hold what the kernels exchange between their workgroups:
 * the draft kernels' ticket counters and tagged router-result slots, the verify call's arrival
 * counters, and the draft status word.  Both calls expect the counters and tags zero on entry and
 * leave them zero on exit (also when the call is replayed from a HIP graph); nothing else is
 * carried from call to call. */
int moe_workspace_init(moe_ctx *ctx, void *workspace, size_t workspace_bytes, void *stream);

/* Size of the leading part of a workspace that holds the "idle state": 512 bytes of counters and
 * the status word, all zero whenever no call is running, then 16-byte router-exchange slots
 * {8 bytes of logit, 8 bytes of tag} whose tags are zero then.  It does not depend on the token
 * count. */
int moe_workspace_idle_bytes(const moe_layer_desc *desc, size_t *bytes);

/* Outcome of the draft calls that used `workspace` since its last moe_workspace_init. */
#define MOE_DRAFT_OK          0
#define MOE_DRAFT_TIMED_OUT   1
/*
 * Inside a draft launch the workgroups that reduce the router rows hand the logits to all others,
 * which poll for them a bounded number of times (moe_set_draft_spin_limit; default 2^22 polls,
 * seconds).  The wait ends only if the producing workgroups run while the others poll.  The
 * library checks on the host that the launch fits the device at once (else the call returns
 * MOE_ERR_INVALID_ARG), which is enough on a device that runs nothing else; kernels of other
 * streams or processes that hold compute units can delay the producers.  If a workgroup runs out of
 * polls it skips its work: the call still returns MOE_OK (the launch was enqueued), ids_out holds
 * -1 (conf_out 0), y is unspecified, the status word in the workspace is set and stays set, and the
 * counters may be left non-zero.  moe_draft_status waits for `stream`, reads the word and writes
 * MOE_DRAFT_OK or MOE_DRAFT_TIMED_OUT to *status (HOST pointer).  After a time-out call
 * moe_workspace_init before the workspace is used again.  (moe_draft_layer_int4_noalloc clears its
 * scratch on every call; its status is not kept.)
 */
int moe_set_draft_spin_limit(moe_ctx *ctx, uint32_t polls);          /* polls >= 1 */
int moe_draft_status(moe_ctx *ctx, const void *workspace, size_t workspace_bytes,
                     int32_t *status, void *stream);

/* ---- router: softmax + top-k, histogram, permutation --------------------------------- */

/*
 * Section 2.1 (a router yields a distribution over the experts and the top-k are selected,
 * their outputs weighted by the router scores), section 3.3.1 (each lookahead entry is an
 * expert id with a confidence score from the gating logits), section 3.4.4 (tokens of one
 * expert are made contiguous before verification).
 *
 *   l[t,e] = sum_h x[t,h] w_router[e,h] (+ router_bias[e]),  accumulated in fp64
 *   topk_ids[t,:]  = the k largest logits of token t, descending; equal logits -> lower
 *                    expert index first
 *   topk_conf[t,j] = softmax(l[t,:])[topk_ids[t,j]]
 *   topk_w[t,j]    = topk_conf[t,j] / sum_j topk_conf[t,j] if desc->renormalize else topk_conf
 *   counts[e]      = number of assignments a with topk_ids[a] == e
 *   offsets        = exclusive prefix sum of counts, offsets[E] = T * k
 *   perm           = assignment indices sorted by expert, ascending a inside one expert
 *
 * x [T,H] bf16 row-major; w_router [E,H] bf16 row-major; router_bias [E] fp32 or NULL.
 * topk_ids [T,k] int32 and topk_w [T,k] fp32 are required; topk_conf [T,k] fp32, counts [E],
 * offsets [E+1], perm [T*k] (int32) may each be NULL (counts/offsets/perm: all or none).
 * Pointers 16-byte aligned (x, w_router) / 4-byte aligned (the rest).
 */
int moe_route_topk(moe_ctx *ctx, const moe_layer_desc *desc,
                   const void *x_bf16, const void *w_router_bf16, const float *router_bias,
                   int T,
                   int32_t *topk_ids, float *topk_w, float *topk_conf,
                   int32_t *counts, int32_t *offsets, int32_t *perm,
                   void *stream);

/* ---- draft pass ----------------------------------------------------------------------- */

/*
 * Section 3.4.2-3.4.3: the draft model keeps the gate and the shared experts in 16 bit and
 * runs every routed expert from 4-bit group-quantised weights in one fused pass; section
 * 3.3.1: it records (expert id, confidence) per token and layer for the lookahead buffer.
 *
 *   route as in moe_route_topk, then
 *   y[t] = sum_j w[t,j] FFN_{ids[t,j]}(x[t]) + sum_s FFN_shared_s(x[t])
 *   FFN(x) = Wd ( silu(Wg x) (.) (Wu x) ),  routed experts with W = (q - z) * s,
 *   products accumulated in fp32, the intermediate carried with 16 significant bits,
 *   y written as fp32.
 *
 * routed: the E int4 experts (struct above).  shared_bf16: S contiguous bf16 expert blobs, or
 * NULL when desc->n_shared == 0.  1 <= T <= MOE_MAX_DRAFT_TOKENS (the canonical call is
 * T = 1; with T > 1 each distinct expert's weights are still streamed once).
 * y_f32 [T,H]; ids_out [T,k] int32 in rank order; conf_out [T,k] fp32 or NULL.  ids_out /
 * conf_out may point into a larger [step, layer, T, k] buffer so that a whole window can be
 * copied to the host at once (section 4.1.2, batched device-to-host transfer).
 * `workspace` must be in its idle state (moe_workspace_init once; every draft call restores
 * it).  y is summed with fp32 atomics, so its last bits may differ from run to run; ids and
 * confidences do not.  ids_out = -1 marks a call whose bounded wait ran out (moe_draft_status).
 * Returns MOE_ERR_INVALID_ARG also when the launch would not fit the device at once.
 */
int moe_draft_layer_int4(moe_ctx *ctx, const moe_layer_desc *desc,
                         const void *x_bf16, const void *w_router_bf16,
                         const float *router_bias,
                         const moe_int4_experts *routed, const void *shared_bf16,
                         int T,
                         float *y_f32, int32_t *ids_out, float *conf_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_draft_layer_int4 for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * mathematics and outputs as moe_draft_layer_int4 minus the workspace: the scratch is a static
 * device array inside the library, moe_noalloc_scratch_bytes() = 2 MiB per GPU, held until the
 * process ends.  The call allocates nothing (no hipMalloc / hipFree, no event creation: launches
 * of this call are never given profiling event pairs) and enqueues a fill kernel that clears the
 * part of the array the draft kernel needs zero, then the launches of moe_draft_layer_int4.
 * Shapes whose workspace (moe_workspace_bytes(desc, T)) exceeds the array return
 * MOE_ERR_WORKSPACE with nothing enqueued; the context's device must be the current device
 * (else MOE_ERR_INVALID_ARG).  All calls on one GPU share the one array: calls that overlap on a
 * GPU (two streams, two contexts) race; order them on one stream or with events.
 */
size_t moe_noalloc_scratch_bytes(void);
int moe_draft_layer_int4_noalloc(moe_ctx *ctx, const moe_layer_desc *desc,
                                 const void *x_bf16, const void *w_router_bf16,
                                 const float *router_bias,
                                 const moe_int4_experts *routed, const void *shared_bf16,
                                 int T,
                                 float *y_f32, int32_t *ids_out, float *conf_out,
                                 void *stream);

/*
 * The draft model over a long run of tokens (the prompt).  Section 3.4.2-3.4.3 describe the
 * int4 layer and choose its backend for the prefill stage as well as the decode stage (the
 * figure comparing backends there).  Same mathematics, arguments and outputs as moe_draft_layer_int4 for 1 <= T <=
 * MOE_MAX_PREFILL_TOKENS tokens.  All tokens are routed first, the assignments are grouped by
 * expert and cut into work items of up to 64, and every expert's weights are streamed once per
 * item (a token-by-token loop streams them once per assignment): a gate/up contraction per
 * (item, 64 intermediate rows) leaves h in the workspace, a down contraction per (item, 128
 * output rows) leaves each assignment's output there, and a last kernel adds up a token's k
 * outputs in assignment order.  No kernel adds into memory that another workgroup writes, so
 * y does not depend on the order in which workgroups run.  Shared experts run over chunks of
 * up to 16 tokens and are added last.
 * ids_out [T,k] and conf_out [T,k] (or NULL) as in moe_draft_layer_int4; y_f32 [T,H] is written.
 * workspace: moe_prefill_workspace_bytes(desc, T) bytes (it grows with T k (3 H + 2 I) x 2 bytes
 * for the operand tiles and outputs of the items), 256-byte aligned, no state is kept in it
 * between calls.
 */
int moe_prefill_workspace_bytes(const moe_layer_desc *desc, int T, size_t *bytes);
int moe_draft_prefill_int4(moe_ctx *ctx, const moe_layer_desc *desc,
                           const void *x_bf16, const void *w_router_bf16,
                           const float *router_bias,
                           const moe_int4_experts *routed, const void *shared_bf16,
                           int T,
                           float *y_f32, int32_t *ids_out, float *conf_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---- union of the experts of a speculative window -------------------------------------- */

/*
 * Section 2.3: verification must load and compute the union of the experts of all tokens of
 * the window; section 3.2.2: the experts still to be fetched, E_new, are that union minus
 * the cache contents.
 *
 * ids [n_ids] int32 (any shape flattened, values in [0, n_experts)), n_ids >= 0.
 * slot_of_expert [n_experts] int32 (-1 = not resident) or NULL.
 * mask [ceil(n_experts / 64)] uint64: bit e set iff e occurs.  list [n_experts]: the
 * distinct ids ascending (first *n_list entries valid).  missing [n_experts] / n_missing:
 * the listed experts whose slot is negative, ascending; with slot_of_expert == NULL
 * *n_missing = 0 and `missing` may be NULL.  All outputs are device memory.
 */
int moe_expert_union(moe_ctx *ctx, const int32_t *ids, int n_ids, int n_experts,
                     const int32_t *slot_of_expert,
                     uint64_t *mask, int32_t *list, int32_t *n_list,
                     int32_t *missing, int32_t *n_missing, void *stream);

/* ---- verify pass ------------------------------------------------------------------------ */

/*
 * Section 3.4.4 and section 2.3: the target model's MoE layer over the K+1 tokens of the
 * window in 16 bit, tokens regrouped per expert so that every distinct expert's weights are
 * streamed once, experts read from the VRAM expert cache.
 *
 *   route as in moe_route_topk, then y as in the draft pass with bf16 weights, fp32
 *   accumulation, the SwiGLU intermediate rounded to bf16, y rounded to bf16.
 *
 * Expert e lives at slot_pool + slot_of_expert[e] * slot_stride_bytes as one bf16 expert
 * blob; slot_of_expert[e] < 0 means "not resident".  Without flags, the terms of non-resident
 * experts are left out of y and their ids are written to missing[0 .. *n_missing) ascending
 * (the caller fetches them and calls again with MOE_VERIFY_ACCUMULATE |
 * MOE_VERIFY_ONLY_LISTED and the same `missing` / `n_missing`, which then adds exactly those
 * terms -- the on-demand load of section 4.1.2).  With MOE_VERIFY_ONLY_LISTED the shared
 * experts are skipped (the first call already added them) and `missing` / `n_missing` are
 * read, then rewritten with what is still absent.
 * MOE_VERIFY_STRICT: the call waits for the stream and returns MOE_ERR_MISSING_EXPERT if
 * *n_missing != 0 (y is then still the partial sum).
 *
 * 1 <= T <= MOE_MAX_TOKENS.  y_bf16 [T,H]; ids_out [T,k] int32 or NULL; missing [E] int32 and
 * n_missing [1] int32 device memory, required.  `workspace` must have been put into its idle
 * state once (moe_workspace_init): the launch that routes counts its arriving workgroups there
 * and leaves the counter zero again.
 */
int moe_verify_layer_bf16(moe_ctx *ctx, const moe_layer_desc *desc,
                          const void *x_bf16, const void *w_router_bf16,
                          const float *router_bias,
                          const void *slot_pool, size_t slot_stride_bytes,
                          const int32_t *slot_of_expert, const void *shared_bf16,
                          int T, int flags,
                          void *y_bf16, int32_t *ids_out,
                          int32_t *missing, int32_t *n_missing,
                          void *workspace, size_t workspace_bytes, void *stream);

/* ---- expert fetch ------------------------------------------------------------------------ */

/*
 * Section 4.1.2: experts are loaded asynchronously from pinned host memory with non-blocking
 * copies on their own stream, ordered against compute with events.
 *
 * Copies `bytes` from src_pinned_host (HOST pointer, page-locked) to dst_slot_dev on
 * copy_stream and, if done_event is not NULL, records it on copy_stream after the copy.
 * The compute stream must wait on that event before a verify call reads the slot.
 */
int moe_expert_copy_async(moe_ctx *ctx, void *dst_slot_dev, const void *src_pinned_host,
                          size_t bytes, void *copy_stream, void *done_event);

/* ---- measurement aid (not part of the method) ---------------------------------------------- */

#define MOE_KERNEL_ROUTE         0   /* router logits + softmax + top-k; in the verify call the same launch also builds the plan (route_plan_kernel) */
#define MOE_KERNEL_PLAN          1   /* histogram / permutation of moe_route_topk (perm_kernel) */
#define MOE_KERNEL_DRAFT_FUSED   2   /* router + top-k + int4 SwiGLU experts, one launch     */
#define MOE_KERNEL_STREAM_READ   3   /* plain streaming read (moe_stream_read_probe)         */
#define MOE_KERNEL_BF16_GATEUP   4   /* bf16 gate+up small-M contraction, SwiGLU             */
#define MOE_KERNEL_BF16_DOWN     5   /* bf16 down small-M contraction                        */
#define MOE_KERNEL_COMBINE       6   /* weighted sum over a token's experts                  */
#define MOE_KERNEL_UNION         7   /* expert union                                         */
#define MOE_KERNEL_PREFILL_STAGE   8  /* moe_draft_prefill_int4: tokens gathered into operand tiles  */
#define MOE_KERNEL_PREFILL_GATEUP  9  /* ... int4 gate+up grouped small-M contraction, SwiGLU         */
#define MOE_KERNEL_PREFILL_DOWN    10 /* ... int4 down grouped small-M contraction                    */
#define MOE_KERNEL_PREFILL_COMBINE 11 /* ... weighted sum over a token's experts                      */
#define MOE_KERNEL_COUNT         12

/* With profiling enabled, every kernel launch of moe_route_topk / moe_draft_layer_int4 /
 * moe_expert_union / moe_verify_layer_bf16 / moe_stream_read_probe carries a pair of HIP events
 * that the runtime stamps with the begin and the end of the kernel's execution on the call's
 * stream (the duration a kernel trace shows).  Events are created on demand, so this mode
 * allocates and must not be used under stream capture; it exists for benchmarks only.
 * Disabling discards pending pairs. */
int moe_profile_enable(moe_ctx *ctx, int enable);
/* Waits for every recorded pair of `kernel`, returns the summed elapsed time and the number of
 * launches since the last read, and clears them.  total_ms / launches are HOST pointers. */
int moe_profile_read(moe_ctx *ctx, int kernel, double *total_ms, int64_t *launches);
/* Static name of a MOE_KERNEL_* id (the kernel's function name), "" if out of range. */
const char *moe_kernel_name(int kernel);

/*
 * Practical ceiling for the weight-streaming kernels: reads `bytes` of device memory at src_dev
 * once and does nothing else, with `workgroups` workgroups of 512 threads, each wave walking its
 * own contiguous run of 1 KiB tiles with eight 16-byte non-temporal loads in flight per lane (the
 * access shape of the draft kernel's weight stream).  bytes: multiple of 1024, >= 1024; src_dev
 * 16-byte aligned; sink_dev: DEVICE pointer to >= 4 writable bytes (written only if the fold of
 * the data equals one reserved word; never read).  Timed like the other kernels through
 * moe_profile_read(MOE_KERNEL_STREAM_READ).  MOE_ERR_INVALID_ARG on bad arguments.
 */
int moe_stream_read_probe(moe_ctx *ctx, const void *src_dev, size_t bytes, int workgroups,
                          void *sink_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOESPEQ_H */
