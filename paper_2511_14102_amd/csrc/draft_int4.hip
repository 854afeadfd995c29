// Draft-pass kernel for calls of two to eight tokens: router, top-k and the SwiGLU FFN of the
// selected experts on group-wise int4 weights, dequantisation fused into the matrix products, ONE
// launch per call (gfx950).  (A call with one token runs the kernel of draft_slice.hip.)
//
// Paper section 3.4.3: the draft pass has to avoid the launch and utilisation losses of
// per-expert small GEMMs (one monolithic expert-fused kernel); section 4.1.3: 4-bit weights in
// groups along the input dimension; section 3.3.1: (expert id, confidence) per token and layer
// is recorded for the lookahead buffer.  The arithmetic is described in draft_common.h.
//
// Work decomposition.  A work item is (expert, slice of 32 intermediate rows): the 32 gate and
// 32 up pre-activations (K = H split over the waves by groups), h = silu(gate) * up, and at
// once the product of h with the 32 matching columns of the down projection for all H outputs,
// added into y with fp32 atomics.  Nothing but the router result crosses workgroups.
//
// The launch is persistent: the grid never exceeds what the device holds at once, and the items
// are dealt evenly, a run of consecutive items per workgroup.  A wave's weight tiles of all its
// items form ONE stream (gate/up tiles of item 0, its down tiles, gate/up tiles of item 1, ...)
// that is read through a rolling window of tiles in flight, so the loads of an item's successor
// are under way while the item's own sums are reduced, h is formed and its down tiles are
// multiplied.  With several tokens a call has many items (every distinct expert of the call,
// I / 32 slices each) and this wins clearly over one workgroup per item (phi shape, 4 tokens:
// 56 against 76 us, 8 tokens: 90 against 144 us; qwen3 shape, 8 tokens: 60 against 103 us).
// With one token there are about one and a half items per compute unit on the phi shape, a
// workgroup's stream is one or two items long, and there is nothing for it to overlap: 26.3 us
// against 25.5 us for one workgroup per item, the same to 3 % on the other shapes.
//
// Cross-workgroup protocol (one bounded wait, no cache flushes):
//   1. router row e is reduced by workgroup e (mod grid), which first clears its share of y
//      with agent-scope stores, waits for their completion, and then publishes the 16-byte
//      slot {logit, tag = 1} of every token as one 16-byte store (in kReplicas copies);
//   2. every workgroup polls the slots with single 16-byte agent-scope loads until all are
//      tagged, then selects the top-k itself (identical in all workgroups) and draws a ticket;
//   3. y contributions are agent-scope atomics, which land after the clearing stores because
//      the clearing completed before the slots were published;
//   4. the workgroup holding the last ticket (everybody has finished polling by then) clears
//      the tags and the ticket counters at its end, so the workspace is back in its idle state
//      when the kernel ends.  This also holds when the same launch is replayed from a HIP graph.
// The wait of step 2 needs the producing workgroups (the first min(E, grid) ones) to be running
// while the others poll: the grid never exceeds the number of compute units, and a workgroup
// fits a compute unit by itself, so on an otherwise idle device all are resident.  If the wait
// runs out (spin limit), the workgroup skips its items and workgroup 0 reports ids = -1.
#include "draft_common.h"

namespace moespeq {

// Timing-only build (-DMOE_STAMPS, never the shipped library): every wave leaves wall-clock stamps
// (100 MHz) of its phases in a device array that moe_debug_stamps copies out.
#ifdef MOE_STAMPS
__device__ unsigned long long moe_stamps[1024 * 8 * 32];
#define STAMP(id) do { if (lane == 0) moe_stamps[((size_t)blockIdx.x * kWaves + wave) * 32 + (id)] = wall_clock64(); } while (0)
#else
#define STAMP(id) do {} while (0)
#endif

namespace {

// MT: token capacity of the launch (2, 4 or 8; the code also serves 1); UPG: 32-code units per
// group (g / 32); SYM: symmetric format (scale blobs, z = 8); NW: waves of the workgroup; kWin:
// tiles a wave keeps in flight.  (Measured: a tile costs about 70 instructions, most of them in
// dependent chains, and one wave issues such an instruction every 8 to 16 clocks, the scalar ones
// through the one scalar unit all waves of a compute unit share; 16 waves with windows of 4 tiles
// were no faster than 8 waves with windows of 8.)
template <int MT, int UPG, bool SYM, int NW, int kWin>
__global__ __launch_bounds__(NW * 64, (NW / 4) * (MT <= 2 ? 2 : 1))
void draft_stream_kernel(const uint16_t *__restrict__ xin, const FusedArgs a)
{
    constexpr int kWaves = NW, kThreads = NW * 64;   // (these names shadow the 8-wave constants of the prefill kernel)
    constexpr int NI = MT < 4 ? MT : 4;          // D rows (tokens) per lane that can be valid
    constexpr int NC = MT > 4 ? 2 : 1;           // lane groups (of 16) whose D rows can be valid
    __shared__ double s_part[kWaves];
    __shared__ int32_t s_ids[MOE_MAX_ASSIGN];
    __shared__ float s_w[MOE_MAX_ASSIGN];
    __shared__ float s_conf[MOE_MAX_ASSIGN];
    __shared__ unsigned long long s_mask[MOE_MAX_EXPERTS / 64];
    // per-item state is kept twice (item parity): an item's successor is set up while waves may
    // still be reading the item's own
    __shared__ int32_t s_row_a[2][MT];          // assignment index of each row (token slot) of the item
    __shared__ int32_t s_cnt[2];
    __shared__ float s_hsum[2][MT];
    __shared__ int32_t s_flag;
    __shared__ int32_t s_first[2];               // one token, few experts: experts of the first two items
    // partial gate/up sums [wave][row block][token in lane group][lane]
    typedef float red_t[4][NI][NC * 16];
    __shared__ red_t s_red[kWaves];
    __shared__ __attribute__((aligned(16))) uint16_t s_hhi[MT][32], s_hlo[MT][32];
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];   // x copy, its group sums, routing scratch

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T = a.T, H = a.H, E = a.E, I = a.I, k = a.k, g = a.g;
    const int n = T * k;
    const int G = H / g;
    const int xstride = H + 8;                   // bf16 elements per token in LDS (+16 B against bank conflicts)
    uint16_t *s_x = reinterpret_cast<uint16_t *>(s_dyn);
    float *s_xsum = reinterpret_cast<float *>(s_dyn + (size_t)MT * xstride * 2);   // [MT][G]
    // routing scratch behind the group sums, used with many experts: logits [MT][E] (fp64), ranks
    const size_t logit_off = ((size_t)MT * xstride * 2 + (size_t)MT * G * 4 + 7) & ~(size_t)7;
    double *s_logit = reinterpret_cast<double *>(s_dyn + logit_off);
    int32_t *s_rank = reinterpret_cast<int32_t *>(s_dyn + logit_off + (size_t)MT * E * 8);

    STAMP(0);
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
    STAMP(1);
    if (tid == 0) s_flag = 1;
    if (tid < MOE_MAX_EXPERTS / 64) s_mask[tid] = 0ull;
    if (tid < 2 * MT) s_hsum[tid / MT][tid % MT] = 0.f;
    __syncthreads();

    // ---- 1b. (while the router result travels) stage x in LDS and sum it per group
    for (int i = tid; i < T * (H / 8); i += kThreads) {
        const int t = i / (H / 8), c8 = i % (H / 8);
        *reinterpret_cast<u32x4 *>(s_x + t * xstride + c8 * 8) = *reinterpret_cast<const u32x4 *>(xin + (size_t)t * H + c8 * 8);
    }
    __syncthreads();
    for (int i = tid; i < T * G * 16; i += kThreads) {       // 16 threads per (token, group)
        const int part = i & 15, tg_ = i >> 4;
        const int t = tg_ / G, gi = tg_ % G;
        const int per = g / 16;                               // 2, 4 or 8 values each
        const uint16_t *src = s_x + t * xstride + gi * g + part * per;
        float v = 0.f;
        for (int j = 0; j < per; ++j) v += __uint_as_float((uint32_t)src[j] << 16);
        v = wave::row_sum(v);
        if (part == 0) s_xsum[t * G + gi] = v;
    }

    // the u-th distinct expert (u-th set bit of the mask words, which are scalars by then)
    uint32_t mask_lo[MOE_MAX_EXPERTS / 64] = {}, mask_hi[MOE_MAX_EXPERTS / 64] = {};
    auto nth_expert = [&](int u) {
        int seen = 0, expert = 0;
#pragma unroll
        for (int wd = 0; wd < MOE_MAX_EXPERTS / 64; ++wd) {
            unsigned long long mk = ((unsigned long long)mask_hi[wd] << 32) | mask_lo[wd];
            const int pc = __popcll(mk);
            if (u >= seen && u < seen + pc) {
                for (int i = u - seen; i > 0; --i) mk &= mk - 1ull;
                expert = wd * 64 + __ffsll((long long)mk) - 1;
            }
            seen += pc;
        }
        return expert;
    };
    const int nslice = I / 32;
    const int U = H / 32;
    const int r = lane & 15, c = lane >> 4;                  // MFMA lane coordinates
    const UnpackConsts uk = unpack_consts();
    const uint32_t lane_off = (uint32_t)lane * 16u;
    constexpr int kEpl = SYM ? 2 : 1;                        // groups (row tiles) per 256-byte block of entries
    const int nrt = H / 64;
    // ---- this wave's share of every item: gate/up tiles u0 .. u1 (K = H split over the waves by
    // groups; the symmetric format keeps two groups / row tiles in one block of entries: whole
    // pairs per wave), padded to whole windows, then its down row tiles r0 .. r1, padded likewise.
    const int g0 = ((wave * (G / kEpl)) / kWaves) * kEpl, g1 = (((wave + 1) * (G / kEpl)) / kWaves) * kEpl;
    const int u0 = g0 * UPG, u1 = g1 * UPG;
    const int nt = u1 - u0;
    const int ntp = (nt + kWin - 1) / kWin * kWin;
    const int r0 = ((wave * (nrt / kEpl)) / kWaves) * kEpl, r1 = (((wave + 1) * (nrt / kEpl)) / kWaves) * kEpl;
    const int ndw = r1 - r0;
    const int ndp = (ndw + kWin - 1) / kWin * kWin;
    const int Lw = ntp + ndp;                                // stream positions of this wave per item
    // One item: expert and slice, and the addresses of this wave's two runs of tiles.  codes:
    // [gate|up tiles (slice, ku)] then [down tiles (slice, rt)], 64 lanes x 16 B each; scale/zero:
    // [gate|up (slice, group)] then [down (group of I, rt)], one 256-byte block of entries per
    // group (row tile), or per pair of them (symmetric format).
    struct Item {
        const char *szb;
        const char *gu_run, *dn_run;     // this wave's first gate/up tile and first down tile of the slice
        int u, slice, expert;            // u: rank of the expert among the call's distinct experts
    };
    // where item idx sits (no routing needed) ...
    auto item_pos = [&](Item &it, int idx) {
        it.u = idx / nslice;
        it.slice = idx - it.u * nslice;
    };
    auto item_after = [&](Item &it, const Item &prev) {     // ... and its successor, without a division
        const bool wrap = prev.slice + 1 == nslice;
        it.u = wrap ? prev.u + 1 : prev.u;
        it.slice = wrap ? 0 : prev.slice + 1;
    };
    // ... and its addresses, once the experts are known
    auto item_addr = [&](Item &it, int expert) {
        it.expert = expert;
        const char *qb = a.q + (size_t)it.expert * a.stride_q;
        it.szb = a.sz + (size_t)it.expert * a.stride_sz;
        it.gu_run = qb + ((size_t)it.slice * U + u0) * 1024;
        it.dn_run = qb + ((size_t)nslice * U + (size_t)it.slice * nrt + r0) * 1024;
    };
    constexpr bool kOwnGu = MT == 1;       // one token: lane group c finishes row block c only and needs its entry only
    constexpr bool kOwnEntry = MT <= 2;    // down: a lane's D registers hold one row block of every tile

    // Addresses of one window of this wave's stream: kWin positions from q0 (a multiple of kWin,
    // counted from the start of item `cur`; positions from Lw on belong to `nxt`).  Parts are
    // padded to whole windows, so a window lies inside one part: `base` is its first tile and
    // `room` the number of tiles up to the part's end; tile i of the window is tile min(i, room - 1)
    // from base.  EVERY load of the stream is unconditional: past the end of a part it repeats the
    // part's last tile, and past the last item (`more` false) the item's last tile (the compiler
    // counts the loads in flight in program order; a load under a branch makes it wait for more of
    // them than it needs, and a second copy of a loop body without the loads costs a full wait
    // where the copies meet).  One address computation per window, not per tile: the scalar unit
    // is shared by all waves of the compute unit.
    struct Run { const char *base; int room; };
    auto window_run = [&](const Item &cur, const Item &nxt, bool more, int q0) {
        const bool wrap = q0 >= Lw;
        const int qq = wrap ? q0 - Lw : q0;
        const char *gu = wrap ? nxt.gu_run : cur.gu_run, *dn = wrap ? nxt.dn_run : cur.dn_run;
        const int j = qq - ntp;
        Run w;
        w.base = qq < ntp ? gu + (size_t)qq * 1024 : dn + (size_t)j * 1024;
        w.room = qq < ntp ? nt - qq : ndw - j;
        if (wrap && !more) {                                     // nothing follows: repeat the very last tile
            w.base = ndw > 0 ? cur.dn_run + (size_t)(ndw - 1) * 1024 : cur.gu_run + (size_t)(nt > 0 ? nt - 1 : 0) * 1024;
            w.room = 1;
        }
        return w;
    };
    auto tile_of = [&](const Run &w, int i) {
        const int t = i < w.room ? i : w.room - 1;
        return reinterpret_cast<const u32x4 *>(w.base + (size_t)t * 1024 + lane_off);
    };

    // Scale / zero entries do not travel through registers: a wave copies the entries of its own
    // groups and row tiles of an item straight into LDS (16-byte loads that write LDS, 1 KiB per
    // instruction, no destination registers and so nothing the compiler has to keep alive across
    // the item loop) BEFORE it requests any tile of that item.  Vector memory operations complete
    // in order, so once a tile of the item has arrived, so have the item's entries; an entry is
    // read only behind the use of such a tile.  Two copies (item parity): an item's entries are
    // requested while its predecessor's are in use.
    const int ngl = (g1 - g0) / kEpl, ndl = (r1 - r0) / kEpl;          // 256-byte blocks of this wave
    const int gl_max = (G / kEpl + kWaves - 1) / kWaves, dl_max = (nrt / kEpl + kWaves - 1) / kWaves;
    const int eb_gu = (gl_max + 3) / 4 * 1024, eb_dn = (dl_max + 3) / 4 * 1024;
    const size_t ent_off = (logit_off + (size_t)MT * E * 12 + 15) & ~(size_t)15;
    unsigned char *s_ent = s_dyn + ent_off + (size_t)wave * 2 * (eb_gu + eb_dn);   // [parity][gate/up | down]
    const uint32_t s_ent_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)s_ent);   // LDS byte address
    auto request_entries = [&](const Item &it, int par) {
        const uint32_t dst = s_ent_addr + par * (eb_gu + eb_dn);
        const char *gsrc = it.szb + ((size_t)it.slice * (G / kEpl) + g0 / kEpl) * 256;
        for (int op = 0; op * 4 < ngl; ++op) {
            const int off = op * 1024 + (int)lane_off;
            const int lim = ngl * 256 - 16;
            load16_to_lds(gsrc + (off < lim ? off : lim), dst + op * 1024);
        }
        const char *dsrc = it.szb + ((size_t)nslice * (G / kEpl) + (size_t)((it.slice * 32) / g) * (nrt / kEpl) + r0 / kEpl) * 256;
        for (int op = 0; op * 4 < ndl; ++op) {
            const int off = op * 1024 + (int)lane_off;
            const int lim = ndl * 256 - 16;
            load16_to_lds(dsrc + (off < lim ? off : lim), dst + eb_gu + op * 1024);
        }
    };
    // entries of block `unit` (counted from the wave's first), part 0 gate/up, 1 down; `odd`: the
    // second group (row tile) of a pair in the symmetric format
    auto own_entry = [&](int par, int part, int unit, int odd) -> uint32_t {      // this lane's row block c of row r
        const unsigned char *p = s_ent + par * (eb_gu + eb_dn) + part * eb_gu + unit * 256 + r * 16;
        if constexpr (SYM) return *reinterpret_cast<const uint16_t *>(p + odd * 8 + c * 2);
        else return *reinterpret_cast<const uint32_t *>(p + c * 4);
    };
    auto row_entries = [&](int par, int part, int unit, int odd) {                 // all four row blocks of row r
        const unsigned char *p = s_ent + par * (eb_gu + eb_dn) + part * eb_gu + unit * 256 + r * 16;
        GroupParams<SYM> gp;
        if constexpr (SYM) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p + odd * 8);
            gp.w[0] = v.x; gp.w[1] = v.y;
        } else {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(p);
            gp.w[0] = v.x; gp.w[1] = v.y; gp.w[2] = v.z; gp.w[3] = v.w;
        }
        return gp;
    };
    // Orders what follows behind the arrival of a tile: `word` comes from the tile's registers, so
    // the wait for the tile's load precedes this point, and no memory access is moved across it.
    auto behind_tile = [](uint32_t word) { asm volatile("" : : "v"(word) : "memory"); };
    const uint32_t cm1 = 0u - (uint32_t)(c & 1), cm2 = 0u - (uint32_t)(c >> 1);
    auto of_my_block = [&](float v0, float v1, float v2, float v3) {   // v_c, chosen with bit masks
        const uint32_t lo = (__float_as_uint(v1) & cm1) | (__float_as_uint(v0) & ~cm1);
        const uint32_t hi = (__float_as_uint(v3) & cm1) | (__float_as_uint(v2) & ~cm1);
        return __uint_as_float((hi & cm2) | (lo & ~cm2));
    };
    // rows (token slots) of an item: the assignments with its expert, ascending; one wave
    auto item_rows = [&](int expert, int par) {
        int cnt = 0;
        for (int base = 0; base < n; base += 64) {
            const int aidx = base + lane;
            const bool hit = aidx < n && s_ids[aidx] == expert;
            const unsigned long long b = __ballot(hit);
            if (hit) {
                const int pos = cnt + __popcll(b & ((1ull << lane) - 1ull));
                if (pos < MT) s_row_a[par][pos] = aidx;
            }
            cnt += __popcll(b);
        }
        if (lane == 0) s_cnt[par] = cnt < MT ? cnt : MT;
    };

    // Work split: the items (distinct experts ascending, I / 32 slices each) are dealt evenly, n / G
    // each, the first n % G workgroups one more.  With one token the k experts are distinct, so the
    // number of items and this workgroup's positions are known before the routing is, and are
    // computed here, while the router result travels; only the expert numbers are filled in later
    // (on the path from the routing to the first weight load every hundred instructions cost a
    // microsecond: a lone wave issues one dependent instruction every 8 to 16 clocks).
    int it_begin = 0, it_end = 0;
    Item cur, nxt;
    auto split_items = [&](int n_items) {
        const uint32_t it_q = (uint32_t)n_items / gridDim.x, it_r = (uint32_t)n_items - it_q * gridDim.x;
        it_begin = (int)(blockIdx.x * it_q + (blockIdx.x < it_r ? blockIdx.x : it_r));
        it_end = it_begin + (int)it_q + (blockIdx.x < it_r ? 1 : 0);
        item_pos(cur, it_begin);
        if (it_begin + 1 < it_end) item_after(nxt, cur);
        else nxt = cur;
    };
    if constexpr (MT == 1) split_items(k * nslice);

    // ---- 2. wave t polls the slots of token t (bounded), then ranks its logits
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
        STAMP(2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = lane + 64 * i;
            if (e < E) { s_logit[t * E + e] = l[i]; s_rank[t * E + e] = 0; }
        }
        if (E <= kLoneWaveTopk) {
            // Rank of every logit in the strict order (larger first, lower index first among equals),
            // so the ranks are a permutation and rank < k selects.  The wave's 64 lanes are P copies of
            // the experts (E2 = E rounded up to a power of two, P = 64 / E2 >= 2): copy q of expert e
            // counts the logits q per .. q per + per - 1 that come before logit e, read from LDS (the
            // lanes of one copy read one address), and the P counts meet through lane exchanges.  Only
            // the selection is on the path to the first weight load; the softmax follows later.
            int E2 = 2;
            while (E2 < E) E2 <<= 1;
            const int P = 64 / E2, per = (E + P - 1) / P;
            const int q = lane / E2, e = lane % E2;
            const double mine = s_logit[t * E + (e < E ? e : E - 1)];
            int part = 0;
            for (int j = 0; j < per; ++j) {
                const int e2 = q * per + j;
                const double v = s_logit[t * E + (e2 < E ? e2 : E - 1)];
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
            if constexpr (MT == 1) {
                // the experts of this workgroup's first two items, for every wave to pick up behind
                // the barrier (each wave searching the mask by itself keeps the one scalar unit of
                // the compute unit busy for a microsecond)
                unsigned long long sel = __ballot(lane < E && part < k);
                unsigned long long m0 = sel, m1 = sel;
                for (int i = cur.u; i > 0; --i) m0 &= m0 - 1ull;
                for (int i = nxt.u; i > 0; --i) m1 &= m1 - 1ull;
                if (lane == 0) { s_first[0] = __ffsll((long long)m0) - 1; s_first[1] = __ffsll((long long)m1) - 1; }
            }
        }
    }
    // the softmax of wave t's token (few experts), off the path to the first weight load: the
    // selection compared the fp64 logits; the softmax values only have to be good to fp32, so they
    // are computed in fp32 from the fp64 differences
    auto finish_softmax = [&]() {
        if (E > kLoneWaveTopk || wave >= T || s_flag == 0) return;
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
    };
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
    STAMP(3);
    const bool ok = s_flag != 0;
    // This workgroup will not look at the slots again: it will draw a ticket.  The tickets are
    // two-level (kTicketGroups first-level counters, then one) so that the returning atomics do
    // not queue up on one address.  The compiler turns the atomic (one lane, wave-uniform
    // address) into a form whose result it reads back at once, which waits for everything the
    // drawing wave has in flight; before a barrier the whole workgroup would wait for it, so the
    // ticket is drawn behind the barriers of the first item's set-up.
    uint32_t ticket = 0xffffffffu;
    auto draw_ticket = [&]() {
        if (tid == kThreads - 64)
            ticket = __hip_atomic_fetch_add(a.tickets + blockIdx.x % kTicketGroups, 1u, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
    };

    // ---- 3. this workgroup's items: the distinct experts ascending, I / 32 slices each
    int n_experts_used = 0;
#pragma unroll
    for (int wd = 0; wd < MOE_MAX_EXPERTS / 64; ++wd) {
        const unsigned long long mk = s_mask[wd];
        mask_lo[wd] = __builtin_amdgcn_readfirstlane((uint32_t)mk);
        mask_hi[wd] = __builtin_amdgcn_readfirstlane((uint32_t)(mk >> 32));
        n_experts_used += __popc(mask_lo[wd]) + __popc(mask_hi[wd]);
    }
    if constexpr (MT != 1) split_items(ok ? n_experts_used * nslice : 0);
    if (!ok) it_end = it_begin;
    STAMP(14);
    if (it_begin < it_end) {
        if (MT == 1 && E <= kLoneWaveTopk) {
            item_addr(cur, __builtin_amdgcn_readfirstlane(s_first[0]));
            if (it_begin + 1 < it_end) item_addr(nxt, __builtin_amdgcn_readfirstlane(s_first[1]));
            else nxt = cur;
        } else {
            item_addr(cur, nth_expert(cur.u));
            if (it_begin + 1 < it_end) item_addr(nxt, nth_expert(nxt.u));
            else nxt = cur;
        }
        STAMP(15);
        // ---- 3a. the first entries and the first window of weight loads go out before anything
        // else of the item is set up: every microsecond of bookkeeping behind them is hidden by
        // their latency
        u32x4 win[kWin];
        if (Lw > 0) {
            request_entries(cur, 0);
            const Run w0 = window_run(cur, nxt, it_begin + 1 < it_end, 0);
#pragma unroll
            for (int i = 0; i < kWin; ++i) win[i] = __builtin_nontemporal_load(tile_of(w0, i));
        }
        STAMP(4);
        if (wave == 0) item_rows(cur.expert, 0);
        finish_softmax();
        __syncthreads();
        draw_ticket();

        for (int it = it_begin; it < it_end; ++it) {
            const int par = (it - it_begin) & 1;
            const bool last = it + 1 == it_end;
            const int cnt = __builtin_amdgcn_readfirstlane(s_cnt[par]);
            // A-operand row of this lane: token slot r (slots >= cnt repeat slot 0; their D rows are ignored)
            auto lds_row = [&](int slot) { return s_row_a[par][slot] / k; };   // where the slot's x was staged
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
            if (Lw > 0) {
                // the successor's entries, before any of the successor's tiles is requested
                if (!last) request_entries(nxt, par ^ 1);
                u32x4 xa = *reinterpret_cast<const u32x4 *>(xrow + (nt > 0 ? u0 : 0) * 32);
                // one window of the gate/up part; kGuard: some of its tiles may lie past the wave's
                // run (the padding of the last window) and are skipped.  Full windows carry no
                // per-tile tests.
                auto gu_window = [&](int base, auto guarded) {
                    constexpr bool kGuard = decltype(guarded)::value;
                    const Run wr = window_run(cur, nxt, !last, base + kWin);
#pragma unroll
                    for (int i = 0; i < kWin; ++i) {
                        const int pz = base + i, ku = u0 + pz;
                        const u32x4 qv = win[i];
                        // The tile's four words are unpacked first, then the window slot is refilled
                        // (into the registers the words just left: a refill issued earlier would need
                        // other registers and a copy of them, with a full wait, at the loop's head),
                        // then the products.  Left alone, the scheduler gathers the eight refills
                        // behind the whole window's arithmetic.
                        const bf16x8 b0 = unpack8(qv.x, uk), b1 = unpack8(qv.y, uk), b2 = unpack8(qv.z, uk), b3 = unpack8(qv.w, uk);
                        __builtin_amdgcn_sched_barrier(0);
                        win[i] = __builtin_nontemporal_load(tile_of(wr, i));
                        __builtin_amdgcn_sched_barrier(0);
                        if (!kGuard || ku < u1) {
                            const u32x4 xn = *reinterpret_cast<const u32x4 *>(xrow + (ku + 1 < u1 ? ku + 1 : ku) * 32);
                            acc[0] = mfma(xa, b0, acc[0]);
                            acc[1] = mfma(xa, b1, acc[1]);
                            acc[2] = mfma(xa, b2, acc[2]);
                            acc[3] = mfma(xa, b3, acc[3]);
                            xa = xn;
                            if (i % UPG == UPG - 1) {                 // end of a group: scale / zero / offset
                                const int gi = ku / UPG;
                                float xs[NI];
#pragma unroll
                                for (int j = 0; j < NI; ++j) xs[j] = s_xsum[tok[j] * G + gi];
                                behind_tile(qv.x);
                                if constexpr (kOwnGu) {
                                    const uint32_t ev = own_entry(par, 0, (gi - g0) / kEpl, gi & 1);
                                    const float sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(ev & 0xffff));
                                    const float zp = SYM ? 136.f : (float)__builtin_bit_cast(_Float16, (uint16_t)(ev >> 16)) + 128.f;
                                    tot1 += sc * (of_my_block(acc[0][0], acc[1][0], acc[2][0], acc[3][0]) - zp * xs[0]);
#pragma unroll
                                    for (int d = 0; d < 4; ++d) acc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
                                } else {
                                    const GroupParams<SYM> gp = row_entries(par, 0, (gi - g0) / kEpl, gi & 1);
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
                };
                {
                    int base = 0;
                    for (; base + kWin <= nt; base += kWin) gu_window(base, std::false_type{});
                    if (base < ntp) gu_window(base, std::true_type{});
                }
                // the window now holds this wave's first down tiles (or, for a wave without down
                // tiles, the successor's first gate/up tiles)
            }
            if (it - it_begin < 2) STAMP(5 + 4 * (it - it_begin));
            if constexpr (kOwnGu) {
                s_red[wave][c][0][r] = tot1;
            } else if (c < NC) {
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int i = 0; i < NI; ++i) s_red[wave][d][i][c * 16 + r] = tot[d][i];
            }
            __syncthreads();
            if (it - it_begin < 2) STAMP(6 + 4 * (it - it_begin));
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
                    if ((lr & 15) == 0) atomicAdd(&s_hsum[par][slot], hs);
                }
            }
            // the last wave (it has no part in the sums above) sets up the successor's rows and
            // clears the successor's h sums; the other copy of both is still being read
            if (wave == kWaves - 1) {
                if (!last) item_rows(nxt.expert, par ^ 1);
                if (lane < MT) s_hsum[par ^ 1][lane] = 0.f;
            }
            __syncthreads();
            if (it - it_begin < 2) STAMP(7 + 4 * (it - it_begin));

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
            if (Lw > 0 && ndw > 0) {
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
                    const int arow = s_row_a[par][slot];
                    live[i] = t < cnt;
                    hsum[i] = s_hsum[par][slot];
                    tokd[i] = arow / k;
                    rwd[i] = s_w[arow];
                }
                if (it == it_begin) STAMP(16);
                // one pass over the window; every slot is refilled with the stream's tile kWin further
                // on (clamped, unconditional), which after this item's last down tile is the
                // successor's first gate/up tile
                auto down_pass = [&](int j0) {
                    const Run wr = window_run(cur, nxt, !last, ntp + j0 + kWin);
#pragma unroll
                    for (int i = 0; i < kWin; ++i) {
                        const int rt = r0 + j0 + i;
                        const u32x4 qv = win[i];
                        bf16x8 b[4];
                        b[0] = unpack8(qv.x, uk); b[1] = unpack8(qv.y, uk); b[2] = unpack8(qv.z, uk); b[3] = unpack8(qv.w, uk);
                        __builtin_amdgcn_sched_barrier(0);
                        win[i] = __builtin_nontemporal_load(tile_of(wr, i));
                        __builtin_amdgcn_sched_barrier(0);
                        if (it == it_begin) STAMP(17 + i);
                        if (rt < r1) {
                            behind_tile(qv.x);
                            uint32_t ev = 0;
                            GroupParams<SYM> gp;
                            if constexpr (kOwnEntry) ev = own_entry(par, 1, (rt - r0) / kEpl, rt & 1);
                            else gp = row_entries(par, 1, (rt - r0) / kEpl, rt & 1);
#pragma unroll
                            for (int q = 0; q < 4 / kBpa; ++q) {
                                f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int bl = 0; bl < kBpa; ++bl) o = mfma(hab[bl], b[q * kBpa + bl], o);
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
                };
                for (int j0 = 0; j0 < ndw; j0 += kWin) down_pass(j0);
            }
            if (it - it_begin < 2) STAMP(8 + 4 * (it - it_begin));
            cur = nxt;
            if (it + 2 < it_end) { item_after(nxt, cur); item_addr(nxt, nth_expert(nxt.u)); }
        }
    } else {
        finish_softmax();
        draw_ticket();
    }

    STAMP(13);
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

__global__ __launch_bounds__(256)
void zero_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

// Plain streaming read of `tiles` 1 KiB tiles with the access shape of the weight stream above:
// every wave owns a contiguous run of tiles, a lane takes 16 bytes of a tile, kWin non-temporal
// loads in flight per lane, every load unconditional (past the end of the run it repeats the
// last tile: a load under a branch would make the compiler drain the window at every step).
// The words are folded so that the loads cannot be dropped; the fold is stored only when it
// equals a value that memory holding real data will not produce.
template <int kWin>
__global__ __launch_bounds__(512, 2)
void stream_read_kernel(const u32x4 *__restrict__ src, size_t tiles, uint32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const size_t nwaves = (size_t)gridDim.x * 8;
    const size_t wave = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6);
    const size_t per = (tiles + nwaves - 1) / nwaves;
    const size_t first = wave * per;
    const size_t mine = first >= tiles ? 0 : (tiles - first < per ? tiles - first : per);
    if (mine == 0) return;
    const u32x4 *q = src + first * 64 + lane;
    u32x4 win[kWin];
    uint32_t fold = 0;
#pragma unroll
    for (int i = 0; i < kWin; ++i) win[i] = __builtin_nontemporal_load(q + ((size_t)i < mine ? (size_t)i : mine - 1) * 64);
    for (size_t b = 0; b < mine; b += kWin) {
#pragma unroll
        for (int i = 0; i < kWin; ++i) {
            const size_t t = b + i;
            const u32x4 v = win[i];
            const size_t nx = t + kWin < mine ? t + kWin : mine - 1;
            win[i] = __builtin_nontemporal_load(q + nx * 64);
            if (t < mine) fold ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    }
    if (fold == 0x9E3779B9u) sink[0] = fold;
}

// waves per workgroup and window depth for a token capacity
// Launch shape for a token capacity (two tokens: two workgroups may share a compute unit, which
// needs 128 registers per wave; more tokens need more registers and own the unit).  Measured on
// the phi shape, 2 tokens: 37.9 us against 40.7 us with 16 waves and windows of 4.
constexpr int stream_waves(int) { return 8; }
constexpr int stream_window(int) { return 8; }
constexpr int stream_wg_per_cu(int MT) { return MT <= 2 ? 2 : 1; }

// dynamic LDS: the bf16 copy of x (padded rows), its per-group sums, the routing scratch (fp64
// logits and ranks), and per wave two copies of the scale / zero entries of its groups and row
// tiles of one item (whole KiB each)
size_t draft_dynamic_lds(int MT, int H, int g, int E, bool sym)
{
    const int nw = stream_waves(MT);
    size_t lds = ((size_t)MT * (H + 8) * 2 + (size_t)MT * (H / g) * 4 + 7) & ~(size_t)7;
    lds += (size_t)MT * E * 12;
    lds = (lds + 15) & ~(size_t)15;
    const int epl = sym ? 2 : 1;
    const int gl_max = (H / g / epl + nw - 1) / nw, dl_max = (H / 64 / epl + nw - 1) / nw;
    lds += (size_t)nw * 2 * ((size_t)((gl_max + 3) / 4) + (size_t)((dl_max + 3) / 4)) * 1024;
    return lds;
}

template <int MT, bool SYM>
void launch_stream_t(const uint16_t *x, const FusedArgs &a, int n_cu, hipStream_t st)
{
    constexpr int NW = stream_waves(MT), KW = stream_window(MT);
    // at most one workgroup per compute unit, never more than there can be items
    const int maxu = a.E < a.T * a.k ? a.E : a.T * a.k;
    const long items = (long)maxu * (a.I / 32);
    const long slots = (long)n_cu * stream_wg_per_cu(MT);
    const dim3 grid((unsigned)(items < slots ? items : slots)), block(NW * 64);
    const size_t lds = draft_dynamic_lds(MT, a.H, a.g, a.E, SYM);
    if (a.g == 32) launch_with_lds(draft_stream_kernel<MT, 1, SYM, NW, KW>, grid, block, lds, st, x, a);
    else if (a.g == 64) launch_with_lds(draft_stream_kernel<MT, 2, SYM, NW, KW>, grid, block, lds, st, x, a);
    else launch_with_lds(draft_stream_kernel<MT, 4, SYM, NW, KW>, grid, block, lds, st, x, a);
}

template <bool SYM>
void launch_stream(int T, const uint16_t *x, const FusedArgs &a, int n_cu, hipStream_t st)
{
    if (T <= 2) launch_stream_t<2, SYM>(x, a, n_cu, st);
    else if (T <= 4) launch_stream_t<4, SYM>(x, a, n_cu, st);
    else launch_stream_t<8, SYM>(x, a, n_cu, st);
}

}  // namespace

void launch_draft_fused(const Shape &s, const DraftFusedArgs &d, int n_cu, hipStream_t st)
{
    // One token: items are few (k I / 32, about one and a half per compute unit on the phi shape) and
    // one workgroup per item is as fast or a little faster (phi 25.5 us against 26.3 us for the
    // persistent launch, mixtral 49.7 / 50.6, qwen3 18.9 / 19.5); from two tokens on the persistent
    // launch wins (4 tokens: 56 against 76 us, 8 tokens: 90 against 144 us).
    if (s.T == 1) { launch_draft_one_token(s, d, st); return; }
    const FusedArgs a = fused_args(s, d);
    const uint16_t *x = (const uint16_t *)d.x;
    if (d.symmetric) launch_stream<true>(s.T, x, a, n_cu, st);
    else launch_stream<false>(s.T, x, a, n_cu, st);
}

template <int MT, bool SYM>
int stream_resident_per_cu(const Shape &s)
{
    constexpr int NW = stream_waves(MT), KW = stream_window(MT);
    const size_t lds = draft_dynamic_lds(MT, s.H, s.g, s.E, SYM);
    if (s.g == 32) return resident_per_cu(draft_stream_kernel<MT, 1, SYM, NW, KW>, NW * 64, lds);
    if (s.g == 64) return resident_per_cu(draft_stream_kernel<MT, 2, SYM, NW, KW>, NW * 64, lds);
    return resident_per_cu(draft_stream_kernel<MT, 4, SYM, NW, KW>, NW * 64, lds);
}

// The launch shapes: one token, one workgroup per item, dispatched in order, so the first
// min(E, grid) of them are resident together when that many fit on the device at once; more tokens,
// a grid of at most stream_wg_per_cu workgroups per compute unit, all of which must fit at once.
bool draft_producers_resident(const Shape &s, const DraftFusedArgs &d, int n_cu)
{
    const int maxu = s.E < s.T * s.k ? s.E : s.T * s.k;
    const long items = (long)maxu * (s.I / 32);
    if (s.T == 1) {
        const long need = s.E < items ? s.E : items;
        return need <= draft_one_token_resident(s, d, n_cu);
    }
    const int MT = s.T <= 2 ? 2 : (s.T <= 4 ? 4 : 8);
    int per = 0;
    if (d.symmetric) per = MT == 2 ? stream_resident_per_cu<2, true>(s) : (MT == 4 ? stream_resident_per_cu<4, true>(s) : stream_resident_per_cu<8, true>(s));
    else per = MT == 2 ? stream_resident_per_cu<2, false>(s) : (MT == 4 ? stream_resident_per_cu<4, false>(s) : stream_resident_per_cu<8, false>(s));
    return per >= stream_wg_per_cu(MT);
}

bool draft_fits(const Shape &s, int tokens, bool sym)
{
    if (tokens <= 1) return draft_one_token_fits(s);
    const int MT = tokens <= 2 ? 2 : (tokens <= 4 ? 4 : 8);
    // 160 KiB of LDS per workgroup, 20 KiB of them for the kernel's static arrays
    return draft_dynamic_lds(MT, s.H, s.g, s.E, sym) <= (size_t)(160 - 20) * 1024;
}

void launch_stream_read(const void *src, size_t bytes, int workgroups, void *sink, hipStream_t st)
{
    launch(stream_read_kernel<8>, dim3(workgroups), dim3(512), 0, st, (const u32x4 *)src,
                       bytes / 1024, (uint32_t *)sink);
}

#ifdef MOE_STAMPS
extern "C" int moe_debug_stamps(unsigned long long *host, size_t n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(moe_stamps), n * sizeof(unsigned long long), 0, hipMemcpyDeviceToHost);
}
extern "C" int moe_debug_clear_stamps(void)
{
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(moe_stamps)) != hipSuccess) return -1;
    return (int)hipMemset(p, 0, sizeof(unsigned long long) * 1024 * 8 * 32);
}
#endif

void launch_zero(void *p, size_t bytes, hipStream_t st)
{
    const size_t n = bytes / 4;
    int blocks = (int)((n + 255) / 256);
    blocks = blocks > 1024 ? 1024 : (blocks < 1 ? 1 : blocks);
    launch(zero_kernel, dim3(blocks), dim3(256), 0, st, (uint32_t *)p, n);
}

}  // namespace moespeq
