// Draft pass over a long run of tokens (gfx950): the int4 experts as a grouped small-M
// contraction (paper section 3.4.3, the prefill side of the prefill / decode split; int4 weights
// of section 4.1.3).  The tokens are routed first; every expert's assignments are cut into work
// items of up to 64, and each expert's weights are streamed once per item:
//
//   prefill_plan_kernel    assignments sorted by expert, items, slot of every assignment
//   prefill_stage_kernel   the items' tokens gathered into MFMA operand tiles (zero padded), and
//                          the sum of each tile row (32 inputs), which the zero points need
//   prefill_tile_kernel<gate/up>  one workgroup per (item, two slices of 32 intermediate rows):
//                          per slice 64 pre-activations (32 gate, 32 up) x 64 tokens over all of
//                          H, h = silu(gate) * up written as operand tiles of a bf16 value and
//                          its bf16 remainder, plus the tile row sums of h
//   prefill_tile_kernel<down>     one workgroup per (item, two tiles of 64 output rows): those
//                          rows x 64 tokens over all of I, written to a per-slot fp32 buffer
//   prefill_combine_kernel y[t] = sum over the token's k assignments of weight x slot output
//
// No kernel adds into memory another workgroup writes: every output element has one owner, so
// the result does not depend on the order in which workgroups run.
//
// The tile kernel.  Its four waves each own one block of 16 weight rows in each of the
// workgroup's 64-row weight tiles (the dword of that block in every lane's 16 bytes of a code
// tile) and all four token blocks; the token operand tiles of a stage of k-steps are staged
// through LDS once and read by all four waves (LDS double buffered, one barrier per stage; two
// stages of global loads in flight).  Arithmetic as in the other draft kernels:
// codes become the exact bf16 integers 128 + q, a group's products are summed by the matrix cores
// (16x16x32 bf16, fp32 accumulate), and scale, zero point and the 128 offset are applied once per
// group with the sum of the group's activations:  s * (acc - (z + 128) * sum).
#include <hip/hip_runtime.h>
#include "draft_common.h"

namespace moespeq {

namespace {

constexpr int kItemTokens = kPrefillChunk;        // 64 = four token blocks of 16
constexpr int kTileThreads = 256;

struct TileArgs {
    const char *q, *sz;              // int4 codes / scale(-zero) blobs of the routed experts
    size_t stride_q, stride_sz;
    const PrefillItem *items;
    const int32_t *n_items;
    const char *act0, *act1;         // operand tiles [(item nk + u) 4 + tb] of 1 KiB: x, or h and its remainder
    const float *sums;               // [(item nk + u)][64]: sum of each token's 32 values of tile u
    char *h_hi, *h_lo;               // gate/up: out tiles [(item I/32 + slice) 4 + tb]
    float *h_sums;                   // gate/up: out sums [(item I/32 + slice)][64]
    float *obuf;                     // down: out [item 64 + token][H]
    int H, I, g;
};

// scale / zero entry of weight row (d, r) for group `grp` (gate/up: of slice `tile`; down: of row
// tile `tile`), as the 32-bit {s, z} entry or the 16-bit scale of the symmetric format
template <bool DOWN, bool SYM>
__device__ inline uint32_t load_entry(const char *szb, int H, int I, int g, int tile, int grp, int r, int d)
{
    const size_t gu_entries = (size_t)(I / 32) * (H / g) * 64;
    size_t e;
    if constexpr (!SYM) {
        e = DOWN ? gu_entries + (((size_t)grp * (H / 64) + tile) * 16 + r) * 4 + d
                 : (((size_t)tile * (H / g) + grp) * 16 + r) * 4 + d;
        return reinterpret_cast<const uint32_t *>(szb)[e];
    } else {
        e = DOWN ? gu_entries + ((((size_t)grp * (H / 128) + tile / 2) * 16 + r) * 2 + tile % 2) * 4 + d
                 : ((((size_t)tile * (H / g / 2) + grp / 2) * 16 + r) * 2 + grp % 2) * 4 + d;
        return reinterpret_cast<const uint16_t *>(szb)[e];
    }
}

template <bool DOWN, bool SYM, int KPG, int RB>
__global__ __launch_bounds__(kTileThreads, 2)
void prefill_tile_kernel(TileArgs a, int max_items)
{
    constexpr int NP = DOWN ? 2 : 1;             // operand planes (h and its remainder)
    constexpr int SK = DOWN ? 2 : 4;             // k-steps per stage
    constexpr int NT = SK * NP * 4;              // operand tiles per stage (16 KiB)
    constexpr int GS = KPG < SK ? KPG : SK;      // k-steps per row of sums
    constexpr int NR = SK / GS;                  // rows of sums per stage
    constexpr int kSumsOff = NT * 1024;          // then NR x 64 fp32 sums
    constexpr int kStageBytes = kSumsOff + SK * 256;
    __shared__ __align__(16) unsigned char s_stage[2][kStageBytes];

    // RB weight tiles per workgroup (gate/up: slices; down: row tiles of 64), tile0 the first
    const int item = blockIdx.x % max_items, tile0 = (blockIdx.x / max_items) * RB;
    if (item >= *a.n_items) return;
    const PrefillItem it = a.items[item];
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, c = lane >> 4;
    const int d = __builtin_amdgcn_readfirstlane(tid >> 6);           // this wave's row block in every tile
    const int H = a.H, I = a.I, g = 32 * KPG;
    const int nk = DOWN ? I / 32 : H / 32, nfull = nk / SK;
    const int ntiles = DOWN ? H / 64 : I / 32;
    const UnpackConsts uk = unpack_consts();

    // a tile past the end repeats the last one (its results are dropped)
    auto tile_of = [&](int rb) { return tile0 + rb < ntiles ? tile0 + rb : ntiles - 1; };
    const char *wq = a.q + (size_t)it.expert * a.stride_q + (DOWN ? (size_t)(I / 32) * (H / 32) * 1024 : 0) +
                     lane * 16 + 4 * d;
    auto wstep = [&](int rb, int u) -> size_t {
        return DOWN ? ((size_t)u * (H / 64) + tile_of(rb)) * 1024 : ((size_t)tile_of(rb) * (H / 32) + u) * 1024;
    };
    const char *szb = a.sz + (size_t)it.expert * a.stride_sz;
    const size_t step0 = (size_t)item * nk;
    f32x4 tot[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) tot[rb][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // The whole K loop for an item with NTB token blocks (a compile-time count: no branch inside
    // a stage, so the LDS reads of a stage are issued ahead of its MFMAs).
    // kAct: this wave's token block exists (d < NTB), so it stages operand tiles and sums; the
    // waves of absent blocks only take part in the weights.  Both are compile-time properties of
    // the code a wave runs, and the loads of a stage are unconditional (past the end they repeat
    // the last stage): a load inside a branch makes the compiler wait for ALL loads in flight
    // where the branch joins, which would undo the two-stage pipeline.
    auto run = [&](auto ntb_c, auto act_c) {
        constexpr int NTB = decltype(ntb_c)::value;
        constexpr bool kAct = decltype(act_c)::value;
        // What one thread moves per stage: its wave's token block of every operand tile, the code
        // dword and the entry of its row block for every tile and k-step, and 16 bytes of one
        // sums row (a row adds up the GS k-steps of a group that lie in the stage).  Two stages
        // are in flight: set R[P] is loaded two stages ahead and written to LDS one stage ahead.
        struct Stage { u32x4 act[SK * NP]; uint32_t w[RB][SK], e[RB][SK]; f32x4 sum[GS]; };
        Stage R[2];
        uint32_t cur_w[RB][SK], cur_e[RB][SK];
        const int sum_row = (lane >> 2) & (NR - 1), sum_piece = lane & 3;   // this lane's 16 bytes of the sums
        auto load_stage = [&](int n, Stage &S) {
#pragma unroll
            for (int s = 0; s < SK; ++s) {
                const int u = n * SK + s < nk ? n * SK + s : nk - 1;
                if constexpr (kAct) {
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        S.act[s * NP + p] = *reinterpret_cast<const u32x4 *>(
                            (p == 0 ? a.act0 : a.act1) + ((step0 + u) * 4 + d) * 1024 + lane * 16);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    S.w[rb][s] = *reinterpret_cast<const uint32_t *>(wq + wstep(rb, u));
                    S.e[rb][s] = load_entry<DOWN, SYM>(szb, H, I, g, tile_of(rb), u / KPG, r, d);
                }
            }
            if constexpr (kAct) {
                // sums of this wave's token block: rows lie inside [0, nk) or outside as a whole; added
                // up when they go to LDS (adding here would make the wave wait for the loads)
                const int u0 = n * SK + sum_row * GS < nk ? n * SK + sum_row * GS : nk - GS;
#pragma unroll
                for (int j = 0; j < GS; ++j)
                    S.sum[j] = *reinterpret_cast<const f32x4 *>(a.sums + (step0 + u0 + j) * 64 + 16 * d + 4 * sum_piece);
            }
        };
        auto store_stage = [&](int b, const Stage &S) {
            if constexpr (kAct) {
#pragma unroll
                for (int j = 0; j < SK * NP; ++j)
                    *reinterpret_cast<u32x4 *>(&s_stage[b][(j * 4 + d) * 1024 + lane * 16]) = S.act[j];
                f32x4 v = S.sum[0];
#pragma unroll
                for (int j = 1; j < GS; ++j) v += S.sum[j];
                if (lane < 4 * NR)
                    *reinterpret_cast<f32x4 *>(&s_stage[b][kSumsOff + sum_row * 256 + (16 * d + 4 * sum_piece) * 4]) = v;
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int s = 0; s < SK; ++s) { cur_w[rb][s] = S.w[rb][s]; cur_e[rb][s] = S.e[rb][s]; }
        };
        f32x4 acc[RB][NTB], xs[NTB];
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
            xs[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        auto group_end = [&](int s) {                             // scale, zero point, offset
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const uint32_t ev = cur_e[rb][s];
                const float sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(ev & 0xffff));
                const float zp = SYM ? 136.f : (float)__builtin_bit_cast(_Float16, (uint16_t)(ev >> 16)) + 128.f;
                const float nsz = -sc * zp;
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        tot[rb][tb][i] = fmaf(sc, acc[rb][tb][i], tot[rb][tb][i]);
                        tot[rb][tb][i] = fmaf(nsz, xs[tb][i], tot[rb][tb][i]);
                    }
                    acc[rb][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
                }
            }
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) xs[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
        };
        // the k-steps of stage n from LDS buffer n & 1; full: all SK of them exist
        auto compute_stage = [&](int n, auto full) {
            constexpr bool kFull = decltype(full)::value;
            const unsigned char *buf = s_stage[n & 1];
#pragma unroll
            for (int s = 0; s < SK; ++s) {
                if (kFull || n * SK + s < nk) {
                    bf16x8 wb[RB];
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) wb[rb] = unpack8(cur_w[rb][s], uk);
#pragma unroll
                    for (int tb = 0; tb < NTB; ++tb) {
#pragma unroll
                        for (int p = 0; p < NP; ++p) {
                            const u32x4 xa = *reinterpret_cast<const u32x4 *>(&buf[((s * NP + p) * 4 + tb) * 1024 + lane * 16]);
#pragma unroll
                            for (int rb = 0; rb < RB; ++rb) acc[rb][tb] = mfma(xa, wb[rb], acc[rb][tb]);
                        }
                        if ((s + 1) % GS == 0)
                            xs[tb] += *reinterpret_cast<const f32x4 *>(&buf[kSumsOff + (s / GS) * 256 + (16 * tb + 4 * c) * 4]);
                    }
                    if constexpr (KPG <= SK) {
                        if ((s + 1) % KPG == 0) group_end(s);
                    } else {
                        if (s == SK - 1 && (n & (KPG / SK - 1)) == KPG / SK - 1) group_end(s);
                    }
                }
            }
        };
        const int ns = (nk + SK - 1) / SK;
        auto iteration = [&](int n, auto parity) {
            constexpr int P = decltype(parity)::value;
            load_stage(n + 2 < ns ? n + 2 : ns - 1, R[P]);
            if (n < nfull) compute_stage(n, std::true_type{});
            else compute_stage(n, std::false_type{});
            if (n + 1 < ns) store_stage((n + 1) & 1, R[P ^ 1]);
            __syncthreads();
        };

        load_stage(0, R[0]);
        load_stage(ns > 1 ? 1 : 0, R[1]);
        store_stage(0, R[0]);
        __syncthreads();
        int n = 0;
        for (; n + 1 < ns; n += 2) {
            iteration(n, std::integral_constant<int, 0>{});
            iteration(n + 1, std::integral_constant<int, 1>{});
        }
        if (n < ns) iteration(n, std::integral_constant<int, 0>{});
    };
    const int ntb = (it.cnt + 15) >> 4;
    auto run_role = [&](auto ntb_c) {
        if (d < decltype(ntb_c)::value) run(ntb_c, std::true_type{});
        else run(ntb_c, std::false_type{});
    };
    if (ntb == 4) run(std::integral_constant<int, 4>{}, std::true_type{});
    else if (ntb == 3) run_role(std::integral_constant<int, 3>{});
    else if (ntb == 2) run_role(std::integral_constant<int, 2>{});
    else run_role(std::integral_constant<int, 1>{});

    // lane (r, c) of wave d now holds, per tile and token block, rows d x 16 + r of tokens 4 c + i
    if constexpr (DOWN) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (tile0 + rb >= ntiles) break;
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int tok = 16 * tb + 4 * c + i;
                    if (tok < it.cnt)
                        a.obuf[((size_t)item * kItemTokens + tok) * H + 64 * (tile0 + rb) + 16 * d + r] = tot[rb][tb][i];
                }
            }
        }
    } else {
        // one slice at a time: pre-activations to LDS as [row block][token][r], then each wave
        // turns one token block into its operand tile: lane (token, chunk) holds h of inputs
        // 8 chunk .. 8 chunk + 7
        float *s_out = reinterpret_cast<float *>(&s_stage[0][0]);       // 16 KiB
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (tile0 + rb >= ntiles) break;                             // the same for the whole workgroup
            if (rb > 0) __syncthreads();
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                if (tb < ntb) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) s_out[(d * 64 + 16 * tb + 4 * c + i) * 16 + r] = tot[rb][tb][i];
                }
            }
            __syncthreads();
            if (d < ntb) {
                const int tok = 16 * d + r;
                uint32_t hi[4], lo[4];
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int col = 8 * c + j, dd = col >> 4, rr = col & 15;
                    const float gate = s_out[(dd * 64 + tok) * 16 + rr], up = s_out[((2 + dd) * 64 + tok) * 16 + rr];
                    const float h = gate / (1.f + expf(-gate)) * up;
                    const uint32_t hb = f32_to_bf16_rne(h);
                    const float rest = h - __uint_as_float(hb << 16);
                    const uint32_t lb = f32_to_bf16_rne(rest);
                    sum += __uint_as_float(hb << 16) + __uint_as_float(lb << 16);
                    if (j & 1) { hi[j >> 1] |= hb << 16; lo[j >> 1] |= lb << 16; }
                    else { hi[j >> 1] = hb; lo[j >> 1] = lb; }
                }
                const size_t slice = (size_t)item * (I / 32) + tile0 + rb;
                const size_t t = (slice * 4 + d) * 1024 + lane * 16;
                *reinterpret_cast<u32x4 *>(a.h_hi + t) = (u32x4){hi[0], hi[1], hi[2], hi[3]};
                *reinterpret_cast<u32x4 *>(a.h_lo + t) = (u32x4){lo[0], lo[1], lo[2], lo[3]};
                sum += __shfl_xor(sum, 16);
                sum += __shfl_xor(sum, 32);
                if (c == 0) a.h_sums[slice * 64 + tok] = sum;
            }
        }
    }
}

// Gathers the tokens of token block (item, tb) into operand tiles [(item nk + u) 4 + tb]: lane
// (token, chunk) of tile u holds x[token][32 u + 8 chunk .. + 7]; positions past the item's count
// hold zeros.  Also the sum of each token's 32 values of the tile.  One wave per (block, u).
__global__ __launch_bounds__(256)
void prefill_stage_kernel(const uint16_t *__restrict__ x, const PrefillItem *__restrict__ items,
                          const int32_t *__restrict__ n_items, const int32_t *__restrict__ sorted,
                          char *__restrict__ xt, float *__restrict__ sums, int H, int k)
{
    const int item = blockIdx.x >> 2, tb = blockIdx.x & 3;
    if (item >= *n_items) return;
    const PrefillItem it = items[item];
    if (16 * tb >= it.cnt) return;
    const int nk = H / 32, u = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (u >= nk) return;
    const int lane = threadIdx.x & 63, tok16 = lane & 15, chunk = lane >> 4, pos = 16 * tb + tok16;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (pos < it.cnt) {
        const int token = sorted[it.first + pos] / k;
        v = *reinterpret_cast<const u32x4 *>(x + (size_t)token * H + 32 * u + 8 * chunk);
    }
    *reinterpret_cast<u32x4 *>(xt + (((size_t)item * nk + u) * 4 + tb) * 1024 + lane * 16) = v;
    float s = ((bf16_lo(v.x) + bf16_hi(v.x)) + (bf16_lo(v.y) + bf16_hi(v.y))) +
              ((bf16_lo(v.z) + bf16_hi(v.z)) + (bf16_lo(v.w) + bf16_hi(v.w)));
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (chunk == 0) sums[((size_t)item * nk + u) * 64 + pos] = s;
}

// Sorts the n = T k assignments by expert (the order inside an expert is arbitrary: no result
// depends on it, a row's sums do not depend on the other rows of its item), cuts every expert's
// run into items of at most 64 and records the slot (item x 64 + position) of every assignment.
// One workgroup.
__global__ __launch_bounds__(1024)
void prefill_plan_kernel(const int32_t *__restrict__ ids, int n, int E,
                         int32_t *__restrict__ sorted, int32_t *__restrict__ slot_of,
                         PrefillItem *__restrict__ items, int32_t *__restrict__ n_items)
{
    __shared__ int32_t s_count[MOE_MAX_EXPERTS], s_off[MOE_MAX_EXPERTS], s_fill[MOE_MAX_EXPERTS],
        s_item0[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += blockDim.x) { s_count[e] = 0; s_fill[e] = 0; }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) atomicAdd(&s_count[ids[i]], 1);
    __syncthreads();
    if (threadIdx.x == 0) {
        int off = 0, item = 0;
        for (int e = 0; e < E; ++e) {
            s_off[e] = off;
            s_item0[e] = item;
            off += s_count[e];
            item += (s_count[e] + kItemTokens - 1) / kItemTokens;
        }
        *n_items = item;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const int e = ids[i];
        const int idx = atomicAdd(&s_fill[e], 1);
        sorted[s_off[e] + idx] = i;
        slot_of[i] = (s_item0[e] + idx / kItemTokens) * kItemTokens + idx % kItemTokens;
    }
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int cnt = s_count[e];
        for (int j = 0; j * kItemTokens < cnt; ++j) {
            PrefillItem it;
            it.expert = e; it.first = s_off[e] + j * kItemTokens;
            it.cnt = cnt - j * kItemTokens < kItemTokens ? cnt - j * kItemTokens : kItemTokens;
            it.pad = 0;
            items[s_item0[e] + j] = it;
        }
    }
}

// y[t][:] = sum_j w[t k + j] * obuf[slot_of[t k + j]][:], j ascending
__global__ __launch_bounds__(256)
void prefill_combine_kernel(const float *__restrict__ obuf, const int32_t *__restrict__ slot_of,
                            const float *__restrict__ w_all, float *__restrict__ y, int H, int k)
{
    const int t = blockIdx.x, col = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (col >= H) return;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < k; ++j) {
        const int a = t * k + j;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(obuf + (size_t)slot_of[a] * H + col);
        const float w = w_all[a];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, v[i], acc[i]);
    }
    *reinterpret_cast<f32x4 *>(y + (size_t)t * H + col) = acc;
}

constexpr int kRowBlocks = 2;                     // weight tiles per workgroup of the tile kernel

template <bool DOWN, bool SYM>
void launch_tile_g(const TileArgs &t, int tiles, int max_items, hipStream_t st)
{
    const int cols = (tiles + kRowBlocks - 1) / kRowBlocks;
    const dim3 grid((unsigned)((size_t)cols * max_items)), block(kTileThreads);
    if (t.g == 32) launch(prefill_tile_kernel<DOWN, SYM, 1, kRowBlocks>, grid, block, 0, st, t, max_items);
    else if (t.g == 64) launch(prefill_tile_kernel<DOWN, SYM, 2, kRowBlocks>, grid, block, 0, st, t, max_items);
    else launch(prefill_tile_kernel<DOWN, SYM, 4, kRowBlocks>, grid, block, 0, st, t, max_items);
}

template <bool DOWN>
void launch_tile(const TileArgs &t, bool sym, int tiles, int max_items, hipStream_t st)
{
    if (sym) launch_tile_g<DOWN, true>(t, tiles, max_items, st);
    else launch_tile_g<DOWN, false>(t, tiles, max_items, st);
}

}  // namespace

PrefillBuffers prefill_buffers(const moe_layer_desc &d, int max_items)
{
    PrefillBuffers b;
    const size_t m = (size_t)max_items;
    b.xt = m * (d.hidden / 32) * 4096;
    b.x_sums = m * (d.hidden / 32) * 256;
    b.h_plane = m * (d.inter / 32) * 4096;
    b.h_sums = m * (d.inter / 32) * 256;
    b.obuf = m * kItemTokens * d.hidden * 4;
    return b;
}

void launch_prefill_plan(const int32_t *ids, int n, int E, int32_t *sorted, int32_t *slot_of,
                         PrefillItem *items, int32_t *n_items, hipStream_t st)
{
    launch(prefill_plan_kernel, dim3(1), dim3(1024), 0, st, ids, n, E, sorted, slot_of, items, n_items);
}

void launch_prefill_stage(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st)
{
    const int nk = s.H / 32;
    launch(prefill_stage_kernel, dim3(max_items * 4, (nk + 3) / 4), dim3(256), 0, st,
           (const uint16_t *)p.x, p.items, p.n_items, p.sorted, (char *)p.xt, p.x_sums, s.H, s.k);
}

static TileArgs tile_args(const Shape &s, const PrefillCall &p)
{
    TileArgs t;
    t.q = (const char *)p.q; t.sz = (const char *)p.sz; t.stride_q = p.stride_q; t.stride_sz = p.stride_sz;
    t.items = p.items; t.n_items = p.n_items;
    t.h_hi = (char *)p.h_hi; t.h_lo = (char *)p.h_lo; t.h_sums = p.h_sums; t.obuf = p.obuf;
    t.H = s.H; t.I = s.I; t.g = s.g;
    return t;
}

void launch_prefill_gateup(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st)
{
    TileArgs t = tile_args(s, p);
    t.act0 = (const char *)p.xt; t.act1 = nullptr; t.sums = p.x_sums;
    launch_tile<false>(t, p.symmetric != 0, s.I / 32, max_items, st);
}

void launch_prefill_down(const Shape &s, const PrefillCall &p, int max_items, hipStream_t st)
{
    TileArgs t = tile_args(s, p);
    t.act0 = (const char *)p.h_hi; t.act1 = (const char *)p.h_lo; t.sums = p.h_sums;
    launch_tile<true>(t, p.symmetric != 0, s.H / 64, max_items, st);
}

void launch_prefill_combine(const Shape &s, const PrefillCall &p, hipStream_t st)
{
    launch(prefill_combine_kernel, dim3(s.T, (s.H / 4 + 255) / 256), dim3(256), 0, st,
           (const float *)p.obuf, p.slot_of, p.w_all, p.y, s.H, s.k);
}

}  // namespace moespeq
