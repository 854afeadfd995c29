// bf16 SwiGLU expert kernels for the verify pass (and for the shared experts of the draft
// pass), gfx950.
//
// Paper section 3.4.4: after regrouping, all tokens of one expert are processed together, so
// an expert's weights are streamed from HBM exactly once per call however many of the K+1
// tokens chose it.  Section 2.3: the cost of verification is the union of the experts.
// With at most 16 tokens per expert the work is a [rows x K] x [K x <=16] contraction: the
// weights are the A operand of the 16x16x32 bf16 MFMA, stored pre-tiled so that one 16-byte
// load per lane fetches a whole A tile, and the tokens are the (zero padded) B operand.
// The kernels are bound by the weight stream; MFMA is idle most of the time by design.
#include "plan.h"

namespace moespeq {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
// Weight pointers come out of the plan as integers; they are device (global) memory.  Saying so
// keeps the loads from being FLAT ones, which count on two counters and force full waits.
typedef const __attribute__((address_space(1))) u32x4 *wptr;

constexpr int kWaves = 4;          // K-split inside a workgroup
constexpr int kUnroll = 8;         // tiles in flight per wave and matrix

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// h[row, i] = silu(Wg x)[i] * (Wu x)[i] for the rows (tokens) of one expert and 16 values of i.
// grid.x = I / 16, grid.y = experts; block = 4 waves splitting K = H.
// kHiLo: also write h - bf16(h) (rounded to bf16) to hb_lo, for callers that need h to ~16 bits.
template <bool kHiLo>
__global__ __launch_bounds__(kWaves * 64)
void bf16_gateup_kernel(const Plan *__restrict__ plan, int first_active,
                        const uint16_t *__restrict__ x, uint16_t *__restrict__ hb,
                        uint16_t *__restrict__ hb_lo, int H, int I)
{
    const int u = first_active + blockIdx.y;
    if (u >= plan->n_active) return;
    const int cnt = plan->act_cnt[u];
    if (cnt == 0) return;
    const int off = plan->act_off[u];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, c = lane >> 4;
    const int U = H / 32;
    const size_t mat = (size_t)(I / 16) * U * 64;              // uint4 per matrix
    const wptr wg = (wptr)(plan->act_w0[u]) + (size_t)blockIdx.x * U * 64 + lane;
    const wptr wu = wg + mat;
    const int tok = n < cnt ? plan->row_tok[off + n] : -1;
    const uint16_t *xrow = x + (size_t)(tok < 0 ? 0 : tok) * H + c * 8;
    const int ku0 = (wave * U) / kWaves, ku1 = ((wave + 1) * U) / kWaves;

    f32x4 cg = {0.f, 0.f, 0.f, 0.f}, cu = {0.f, 0.f, 0.f, 0.f};
    int ku = ku0;
    for (; ku + kUnroll <= ku1; ku += kUnroll) {
        u32x4 a[kUnroll], b[kUnroll], xv[kUnroll];
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            a[i] = __builtin_nontemporal_load(wg + (size_t)(ku + i) * 64);
            b[i] = __builtin_nontemporal_load(wu + (size_t)(ku + i) * 64);
            xv[i] = tok >= 0 ? *reinterpret_cast<const u32x4 *>(xrow + (ku + i) * 32) : (u32x4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            cg = mfma16(a[i], xv[i], cg);
            cu = mfma16(b[i], xv[i], cu);
        }
    }
    for (; ku < ku1; ++ku) {
        u32x4 a = __builtin_nontemporal_load(wg + (size_t)ku * 64);
        u32x4 b = __builtin_nontemporal_load(wu + (size_t)ku * 64);
        u32x4 xv = tok >= 0 ? *reinterpret_cast<const u32x4 *>(xrow + ku * 32) : (u32x4){0u, 0u, 0u, 0u};
        cg = mfma16(a, xv, cg);
        cu = mfma16(b, xv, cu);
    }

    __shared__ float s_red[kWaves][2][4][64];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s_red[wave][0][i][lane] = cg[i];
        s_red[wave][1][i][lane] = cu[i];
    }
    __syncthreads();
    if (wave != 0 || n >= cnt) return;
    uint16_t out[4], out_lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float g = 0.f, v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { g += s_red[w][0][i][lane]; v += s_red[w][1][i][lane]; }
        float h = g / (1.f + expf(-g)) * v;
        out[i] = f32_to_bf16_rne(h);
        if (kHiLo) out_lo[i] = f32_to_bf16_rne(h - __uint_as_float((uint32_t)out[i] << 16));
    }
    // D layout: lane holds rows c*4 .. c*4+3 of column n
    const size_t o = (size_t)(off + n) * I + blockIdx.x * 16 + c * 4;
    *reinterpret_cast<uint2 *>(hb + o) = make_uint2((uint32_t)out[0] | ((uint32_t)out[1] << 16),
                                                    (uint32_t)out[2] | ((uint32_t)out[3] << 16));
    if (kHiLo)
        *reinterpret_cast<uint2 *>(hb_lo + o) = make_uint2((uint32_t)out_lo[0] | ((uint32_t)out_lo[1] << 16),
                                                           (uint32_t)out_lo[2] | ((uint32_t)out_lo[3] << 16));
}

// obuf[row, r] = row_w[row] * (Wd h[row])[r] for 16 values of r.
// grid.x = H / 16, grid.y = experts; block = 4 waves splitting K = I.
// kHiLo: the operand is hb + hb_lo (two MFMAs per tile).  kAddY: instead of writing obuf, add the
// row's outputs to y[token] with fp32 atomics (the draft call's shared experts: y already holds
// the routed experts' sum, itself made of such atomics, so no combine launch is needed).
template <bool kHiLo, bool kAddY>
__global__ __launch_bounds__(kWaves * 64)
void bf16_down_kernel(const Plan *__restrict__ plan, int first_active,
                      const uint16_t *__restrict__ hb, const uint16_t *__restrict__ hb_lo,
                      float *__restrict__ obuf, int H, int I)
{
    const int u = first_active + blockIdx.y;
    if (u >= plan->n_active) return;
    const int cnt = plan->act_cnt[u];
    if (cnt == 0) return;
    const int off = plan->act_off[u];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, c = lane >> 4;
    const int U = I / 32;
    const size_t mat = (size_t)(I / 16) * (H / 32) * 64;
    const wptr wd = (wptr)(plan->act_w0[u]) + 2 * mat + (size_t)blockIdx.x * U * 64 + lane;
    const bool live = n < cnt;
    const size_t hoff = (size_t)(off + (live ? n : 0)) * I + c * 8;
    const uint16_t *hrow = hb + hoff;
    const uint16_t *lrow = kHiLo ? hb_lo + hoff : nullptr;
    const int ku0 = (wave * U) / kWaves, ku1 = ((wave + 1) * U) / kWaves;
    const u32x4 zero = {0u, 0u, 0u, 0u};

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int ku = ku0;
    for (; ku + kUnroll <= ku1; ku += kUnroll) {
        u32x4 a[kUnroll], hv[kUnroll], lv[kUnroll];
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            a[i] = __builtin_nontemporal_load(wd + (size_t)(ku + i) * 64);
            hv[i] = live ? *reinterpret_cast<const u32x4 *>(hrow + (ku + i) * 32) : zero;
            if (kHiLo) lv[i] = live ? *reinterpret_cast<const u32x4 *>(lrow + (ku + i) * 32) : zero;
        }
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            acc = mfma16(a[i], hv[i], acc);
            if (kHiLo) acc = mfma16(a[i], lv[i], acc);
        }
    }
    for (; ku < ku1; ++ku) {
        u32x4 a = __builtin_nontemporal_load(wd + (size_t)ku * 64);
        u32x4 hv = live ? *reinterpret_cast<const u32x4 *>(hrow + ku * 32) : zero;
        acc = mfma16(a, hv, acc);
        if (kHiLo) {
            u32x4 lv = live ? *reinterpret_cast<const u32x4 *>(lrow + ku * 32) : zero;
            acc = mfma16(a, lv, acc);
        }
    }

    __shared__ float s_red[kWaves][4][64];
#pragma unroll
    for (int i = 0; i < 4; ++i) s_red[wave][i][lane] = acc[i];
    __syncthreads();
    if (wave != 0 || !live) return;
    const float rw = plan->row_w[off + n];
    float4 o;
    float *op = &o.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += s_red[w][i][lane];
        op[i] = v * rw;
    }
    if constexpr (kAddY) {
        float *yrow = obuf + (size_t)plan->row_tok[off + n] * H + blockIdx.x * 16 + c * 4;   // obuf is y here
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __hip_atomic_fetch_add(yrow + i, op[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *reinterpret_cast<float4 *>(obuf + (size_t)(off + n) * H + blockIdx.x * 16 + c * 4) = o;
    }
}

// Final sum per token in a fixed order: routed rows by rank j (each summed over the K-splits),
// then shared rows.  grid (ceil(H / 1024), T), 256 threads x 4 columns.
template <bool kOutBf16>
__global__ __launch_bounds__(256)
void combine_kernel(const Plan *__restrict__ plan, const float *__restrict__ routed, int nsplit,
                    const float *__restrict__ obuf, int accumulate, void *__restrict__ y,
                    int T, int H, int k, int S)
{
    __shared__ int32_t s_pos[MOE_MAX_TOPK];
    const int t = blockIdx.y;
    const int n = T * k;
    // row of assignment (t, j): the position of a = t*k + j in perm
    for (int pos = threadIdx.x; pos < n; pos += blockDim.x) {
        int a = plan->perm[pos];
        if (a / k == t) s_pos[a % k] = pos;
    }
    __syncthreads();
    const int h = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (h >= H) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (accumulate) {
        if (kOutBf16) {
            uint2 old = *reinterpret_cast<const uint2 *>((const uint16_t *)y + (size_t)t * H + h);
            acc.x = __uint_as_float(old.x << 16);
            acc.y = __uint_as_float(old.x & 0xffff0000u);
            acc.z = __uint_as_float(old.y << 16);
            acc.w = __uint_as_float(old.y & 0xffff0000u);
        } else {
            acc = *reinterpret_cast<const float4 *>((const float *)y + (size_t)t * H + h);
        }
    }
    for (int j = 0; j < k; ++j) {
        const int pos = s_pos[j];
        if (!plan->row_live[pos]) continue;
        for (int sp = 0; sp < nsplit; ++sp) {
            float4 v = *reinterpret_cast<const float4 *>(routed + ((size_t)sp * n + pos) * H + h);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    for (int s = 0; s < S; ++s) {
        const int pos = n + s * T + t;
        if (!plan->row_live[pos]) continue;
        float4 v = *reinterpret_cast<const float4 *>(obuf + (size_t)pos * H + h);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (kOutBf16) {
        uint2 pk = make_uint2((uint32_t)f32_to_bf16_rne(acc.x) | ((uint32_t)f32_to_bf16_rne(acc.y) << 16),
                              (uint32_t)f32_to_bf16_rne(acc.z) | ((uint32_t)f32_to_bf16_rne(acc.w) << 16));
        *reinterpret_cast<uint2 *>((uint16_t *)y + (size_t)t * H + h) = pk;
    } else {
        *reinterpret_cast<float4 *>((float *)y + (size_t)t * H + h) = acc;
    }
}

}  // namespace

void launch_bf16_gateup(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                        const void *x, void *hb, void *hb_lo, hipStream_t st)
{
    if (n_active_max <= 0) return;
    const dim3 grid(s.I / 16, n_active_max), block(kWaves * 64);
    if (hb_lo)
        launch(bf16_gateup_kernel<true>, grid, block, 0, st, plan, first_active,
                           (const uint16_t *)x, (uint16_t *)hb, (uint16_t *)hb_lo, s.H, s.I);
    else
        launch(bf16_gateup_kernel<false>, grid, block, 0, st, plan, first_active,
                           (const uint16_t *)x, (uint16_t *)hb, (uint16_t *)nullptr, s.H, s.I);
}

void launch_bf16_down(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                      const void *hb, const void *hb_lo, float *obuf, hipStream_t st)
{
    if (n_active_max <= 0) return;
    const dim3 grid(s.H / 16, n_active_max), block(kWaves * 64);
    if (hb_lo)
        launch(bf16_down_kernel<true, false>, grid, block, 0, st, plan, first_active,
                           (const uint16_t *)hb, (const uint16_t *)hb_lo, obuf, s.H, s.I);
    else
        launch(bf16_down_kernel<false, false>, grid, block, 0, st, plan, first_active,
                           (const uint16_t *)hb, (const uint16_t *)nullptr, obuf, s.H, s.I);
}

void launch_bf16_down_add(const Shape &s, const Plan *plan, int first_active, int n_active_max,
                          const void *hb, const void *hb_lo, float *y, hipStream_t st)
{
    if (n_active_max <= 0) return;
    const dim3 grid(s.H / 16, n_active_max), block(kWaves * 64);
    launch(bf16_down_kernel<true, true>, grid, block, 0, st, plan, first_active,
                       (const uint16_t *)hb, (const uint16_t *)hb_lo, y, s.H, s.I);
}

void launch_combine(const Shape &s, const Plan *plan, const float *routed, int nsplit,
                    const float *obuf, int accumulate, int out_bf16, void *y, hipStream_t st)
{
    dim3 grid((s.H + 1023) / 1024, s.T);
    if (out_bf16)
        launch(combine_kernel<true>, grid, dim3(256), 0, st, plan, routed, nsplit, obuf,
                           accumulate, y, s.T, s.H, s.k, s.S);
    else
        launch(combine_kernel<false>, grid, dim3(256), 0, st, plan, routed, nsplit, obuf,
                           accumulate, y, s.T, s.H, s.k, s.S);
}

}  // namespace moespeq
