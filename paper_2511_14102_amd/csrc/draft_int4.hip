// Draft-pass expert kernels: SwiGLU FFN on group-wise int4 weights with the dequantisation
// fused into the matrix-vector products (gfx950).
//
// Paper section 3.4.3: the draft pass must run the quantised experts without the launch and
// utilisation losses of per-expert small GEMMs; section 4.1.3: 4-bit weights in groups along
// the input dimension.  W = (q - z) * s, so for one output row and one group G
//     sum_{c in G} W[c] v[c] = s * ( sum_c q[c] v[c]  -  z * sum_c v[c] ),
// i.e. the inner loop needs only the integer codes: the codes are turned into exact fp16
// integers with two bit operations and one packed fp16 op per pair and fed to the
// fp16-pair dot product with fp32 accumulation; scale and zero are applied once per group.
//
// Mapping: one lane owns one output row ("tile64x32" layout: a wave's 16-byte loads of one
// tile are 1 KiB contiguous), so no cross-lane reduction is needed; the activation values of a
// step are wave-uniform and come through scalar loads.  K is split over the waves of a
// workgroup (and, for the down projection, over several workgroups) and recombined in a fixed
// order.
#include "plan.h"

namespace moespeq {

namespace {

typedef __attribute__((ext_vector_type(2))) _Float16 h2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kGuWaves = 8;       // waves per workgroup (K-split) in the gate/up kernel
constexpr int kDownWaves = 4;     // waves per workgroup in the down kernel
constexpr float kLoScale = 2048.f;        // h = hi + lo / 2048 with hi, lo fp16

__device__ inline h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }

// The 8 codes of one 32-bit word as 4 fp16 pairs (codes 0-1, 2-3, 4-5, 6-7), exact.
// 0x6400 is fp16 1024 with a zero mantissa: or-ing a code into mantissa bits 0-3 gives
// 1024 + q, into bits 4-7 gives 1024 + 16 q.
__device__ inline void unpack8(uint32_t w, h2 out[4]) {
    const uint32_t magic = 0x64006400u;
    const uint32_t t = w >> 8;
    const h2 k1024 = {(_Float16)1024.f, (_Float16)1024.f};
    const h2 k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const h2 k64 = {(_Float16)64.f, (_Float16)64.f};
    out[0] = as_h2((w & 0x000F000Fu) | magic) - k1024;
    out[1] = as_h2((w & 0x00F000F0u) | magic) * k16th - k64;
    out[2] = as_h2((t & 0x000F000Fu) | magic) - k1024;
    out[3] = as_h2((t & 0x00F000F0u) | magic) * k16th - k64;
}

// acc += sum over the 32 codes held in `q` (4 words) of code * v, v = 16 consecutive fp16 pairs
__device__ inline float dot32(u32x4 q, const h2 *__restrict__ v, float acc) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        h2 c[4];
        unpack8(w[d], c);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_fdot2(c[j], v[4 * d + j], acc, false);
    }
    return acc;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Sum of g consecutive fp16 values (g in {32, 64, 128}), same result in every lane.
__device__ inline float group_sum(const _Float16 *__restrict__ v, int g, int lane) {
    float s = 0.f;
    for (int i = lane; i < g; i += 64) s += (float)v[i];
    return wave_sum(s);
}
__device__ inline float group_sum_hilo(const _Float16 *__restrict__ hi, const _Float16 *__restrict__ lo,
                                       int g, int lane) {
    float s = 0.f;
    for (int i = lane; i < g; i += 64) s += (float)hi[i] + (float)lo[i] * (1.f / kLoScale);
    return wave_sum(s);
}

// Gate and up projections of one 64-row slice of the intermediate dimension for the (<= MT)
// tokens of one expert, then h = silu(gate) * up, written as an fp16 hi/lo pair.
// grid.x = I / 64, grid.y = routed experts of the call; block = 8 waves splitting K = H by groups.
template <int MT>
__global__ __launch_bounds__(kGuWaves * 64)
void draft_gateup_kernel(const Plan *__restrict__ plan, int S, const _Float16 *__restrict__ xh,
                         _Float16 *__restrict__ hh, _Float16 *__restrict__ hl, int H, int I, int g)
{
    const int u = S + blockIdx.y;
    if (u >= plan->n_active) return;
    const int cnt = plan->act_cnt[u];
    const int off = plan->act_off[u];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int U = H / 32, G = H / g, upg = g / 32;
    const size_t qmat = (size_t)(I / 64) * U * 64;            // 16-byte units per matrix
    const size_t szmat = (size_t)(I / 64) * G * 64;           // 4-byte units per matrix
    const u32x4 *qg = reinterpret_cast<const u32x4 *>(plan->act_w0[u]) + (size_t)blockIdx.x * U * 64 + lane;
    const u32x4 *qu = qg + qmat;
    const uint32_t *szg = reinterpret_cast<const uint32_t *>(plan->act_w1[u]) + (size_t)blockIdx.x * G * 64 + lane;
    const uint32_t *szu = szg + szmat;

    const _Float16 *xt[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) xt[m] = xh + (size_t)plan->row_tok[off + (m < cnt ? m : 0)] * H;

    float tg[MT], tu[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) { tg[m] = 0.f; tu[m] = 0.f; }

    const int g0 = (wave * G) / kGuWaves, g1 = ((wave + 1) * G) / kGuWaves;
    for (int gi = g0; gi < g1; ++gi) {
        float ag[MT], au[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) { ag[m] = 0.f; au[m] = 0.f; }
        for (int uu = 0; uu < upg; ++uu) {
            const int ku = gi * upg + uu;
            const u32x4 a = __builtin_nontemporal_load(qg + (size_t)ku * 64);
            const u32x4 b = __builtin_nontemporal_load(qu + (size_t)ku * 64);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const h2 *xv = reinterpret_cast<const h2 *>(xt[m] + ku * 32);
                ag[m] = dot32(a, xv, ag[m]);
                au[m] = dot32(b, xv, au[m]);
            }
        }
        const h2 sg = as_h2(szg[(size_t)gi * 64]), su = as_h2(szu[(size_t)gi * 64]);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const float xs = group_sum(xt[m] + gi * g, g, lane);
            tg[m] += (float)sg.x * (ag[m] - (float)sg.y * xs);
            tu[m] += (float)su.x * (au[m] - (float)su.y * xs);
        }
    }

    __shared__ float s_red[kGuWaves][2][MT][64];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        s_red[wave][0][m][lane] = tg[m];
        s_red[wave][1][m][lane] = tu[m];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < MT * 64; i += kGuWaves * 64) {
        const int m = i >> 6, r = i & 63;
        if (m >= cnt) continue;
        float gsum = 0.f, usum = 0.f;
#pragma unroll
        for (int w = 0; w < kGuWaves; ++w) { gsum += s_red[w][0][m][r]; usum += s_red[w][1][m][r]; }
        const float un = plan->x_unscale[plan->row_tok[off + m]];
        gsum *= un;
        usum *= un;
        const float h = gsum / (1.f + expf(-gsum)) * usum;
        const _Float16 hi = (_Float16)h;
        const _Float16 lo = (_Float16)((h - (float)hi) * kLoScale);
        const size_t o = (size_t)(off + m) * I + blockIdx.x * 64 + r;
        hh[o] = hi;
        hl[o] = lo;
    }
}

// Down projection of one 64-row slice of the hidden dimension: part[split, row, r] =
// row_w[row] * sum over this workgroup's share of K = I.  grid.x = H / 64, grid.y = routed
// experts, grid.z = K-splits; block = 4 waves splitting the workgroup's share by groups.
template <int MT>
__global__ __launch_bounds__(kDownWaves * 64)
void draft_down_kernel(const Plan *__restrict__ plan, int S, const _Float16 *__restrict__ hh,
                       const _Float16 *__restrict__ hl, float *__restrict__ part,
                       int H, int I, int g, int n_assign)
{
    const int u = S + blockIdx.y;
    if (u >= plan->n_active) return;
    const int cnt = plan->act_cnt[u];
    const int off = plan->act_off[u];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int U = I / 32, G = I / g, upg = g / 32;
    const size_t qmat = (size_t)(I / 64) * (H / 32) * 64;     // gate (and up) codes, 16-byte units
    const size_t szmat = (size_t)(I / 64) * (H / g) * 64;     // gate (and up) scale-zero, 4-byte units
    const u32x4 *qd = reinterpret_cast<const u32x4 *>(plan->act_w0[u]) + 2 * qmat + (size_t)blockIdx.x * U * 64 + lane;
    const uint32_t *szd = reinterpret_cast<const uint32_t *>(plan->act_w1[u]) + 2 * szmat + (size_t)blockIdx.x * G * 64 + lane;

    const _Float16 *hi[MT], *lo[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const size_t r = (size_t)(off + (m < cnt ? m : 0)) * I;
        hi[m] = hh + r;
        lo[m] = hl + r;
    }
    float tot[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) tot[m] = 0.f;

    const int nw = gridDim.z * kDownWaves;
    const int wi = blockIdx.z * kDownWaves + wave;
    const int g0 = (wi * G) / nw, g1 = ((wi + 1) * G) / nw;
    for (int gi = g0; gi < g1; ++gi) {
        float ah[MT], al[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) { ah[m] = 0.f; al[m] = 0.f; }
        for (int uu = 0; uu < upg; ++uu) {
            const int ku = gi * upg + uu;
            const u32x4 a = __builtin_nontemporal_load(qd + (size_t)ku * 64);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                ah[m] = dot32(a, reinterpret_cast<const h2 *>(hi[m] + ku * 32), ah[m]);
                al[m] = dot32(a, reinterpret_cast<const h2 *>(lo[m] + ku * 32), al[m]);
            }
        }
        const h2 sz = as_h2(szd[(size_t)gi * 64]);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const float hs = group_sum_hilo(hi[m] + gi * g, lo[m] + gi * g, g, lane);
            tot[m] += (float)sz.x * (ah[m] + al[m] * (1.f / kLoScale) - (float)sz.y * hs);
        }
    }

    __shared__ float s_red[kDownWaves][MT][64];
#pragma unroll
    for (int m = 0; m < MT; ++m) s_red[wave][m][lane] = tot[m];
    __syncthreads();
    for (int i = threadIdx.x; i < MT * 64; i += kDownWaves * 64) {
        const int m = i >> 6, r = i & 63;
        if (m >= cnt) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kDownWaves; ++w) v += s_red[w][m][r];
        part[((size_t)blockIdx.z * n_assign + off + m) * H + blockIdx.x * 64 + r] = v * plan->row_w[off + m];
    }
}

template <int MT>
void launch_gateup_t(const Shape &s, const Plan *plan, const void *xh, void *hh, void *hl, hipStream_t st)
{
    const int nexp = s.E < s.T * s.k ? s.E : s.T * s.k;
    hipLaunchKernelGGL(draft_gateup_kernel<MT>, dim3(s.I / 64, nexp), dim3(kGuWaves * 64), 0, st, plan,
                       s.S, (const _Float16 *)xh, (_Float16 *)hh, (_Float16 *)hl, s.H, s.I, s.g);
}

template <int MT>
void launch_down_t(const Shape &s, const Plan *plan, const void *hh, const void *hl, float *part,
                   hipStream_t st)
{
    const int nexp = s.E < s.T * s.k ? s.E : s.T * s.k;
    hipLaunchKernelGGL(draft_down_kernel<MT>, dim3(s.H / 64, nexp, kDraftDownSplit), dim3(kDownWaves * 64),
                       0, st, plan, s.S, (const _Float16 *)hh, (const _Float16 *)hl, part, s.H, s.I, s.g,
                       s.T * s.k);
}

}  // namespace

void launch_draft_gateup(const Shape &s, const Plan *plan, const void *xh, void *hh, void *hl,
                         hipStream_t st)
{
    if (s.T <= 1) launch_gateup_t<1>(s, plan, xh, hh, hl, st);
    else if (s.T <= 2) launch_gateup_t<2>(s, plan, xh, hh, hl, st);
    else if (s.T <= 4) launch_gateup_t<4>(s, plan, xh, hh, hl, st);
    else launch_gateup_t<8>(s, plan, xh, hh, hl, st);
}

void launch_draft_down(const Shape &s, const Plan *plan, const void *hh, const void *hl,
                       float *part, hipStream_t st)
{
    if (s.T <= 1) launch_down_t<1>(s, plan, hh, hl, part, st);
    else if (s.T <= 2) launch_down_t<2>(s, plan, hh, hl, part, st);
    else if (s.T <= 4) launch_down_t<4>(s, plan, hh, hl, part, st);
    else launch_down_t<8>(s, plan, hh, hl, part, st);
}

}  // namespace moespeq
