// Wave-wide (64 lanes) reductions for gfx950 through the data-parallel-primitive lane moves of
// the vector ALU instead of LDS-routed lane permutes: a dependent chain of six permutes costs
// around a thousand cycles, the same chain of DPP moves a few tens.  All results are the same in
// every lane and do not depend on timing (fixed combination order).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moespeq {
namespace wave {

// DPP controls: partner lanes inside a row of 16 lanes
constexpr int kSwap1 = 0xB1;        // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kSwap2 = 0x4E;        // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kHalfMirror = 0x141;  // lane i <-> 7 - i inside each 8 lanes (the other quad)
constexpr int kMirror = 0x140;      // lane i <-> 15 - i inside the row (the other half)

template <int kCtrl>
__device__ inline uint32_t move(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, 0xF, 0xF, false);
}
template <int kCtrl>
__device__ inline float move(float v) { return __uint_as_float(move<kCtrl>(__float_as_uint(v))); }
template <int kCtrl>
__device__ inline int move(int v) { return (int)move<kCtrl>((uint32_t)v); }
template <int kCtrl>
__device__ inline double move(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = move<kCtrl>((uint32_t)b), hi = move<kCtrl>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// value of lane `kLane`, as a wave-uniform value
template <int kLane>
__device__ inline uint32_t from_lane(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, kLane); }
template <int kLane>
__device__ inline float from_lane(float v) { return __uint_as_float(from_lane<kLane>(__float_as_uint(v))); }
template <int kLane>
__device__ inline int from_lane(int v) { return __builtin_amdgcn_readlane(v, kLane); }
template <int kLane>
__device__ inline double from_lane(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = from_lane<kLane>((uint32_t)b), hi = from_lane<kLane>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// value of lane `lane` (wave-uniform, not a compile-time constant)
__device__ inline double from_lane(double v, int lane) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Reduction over each row of 16 lanes with a commutative `op`; every lane of the row gets the
// row's result.  After the two quad steps a quad's lanes agree, so the mirror moves pair
// disjoint, already reduced groups.
template <typename T, typename Op>
__device__ inline T row_all(T v, Op op) {
    v = op(v, move<kSwap1>(v));
    v = op(v, move<kSwap2>(v));
    v = op(v, move<kHalfMirror>(v));
    v = op(v, move<kMirror>(v));
    return v;
}

// Reduction over the wave: rows first, then the four row results in row order.
template <typename T, typename Op>
__device__ inline T all(T v, Op op) {
    v = row_all(v, op);
    return op(op(op(from_lane<0>(v), from_lane<16>(v)), from_lane<32>(v)), from_lane<48>(v));
}

__device__ inline float sum(float v) { return all(v, [](float a, float b) { return a + b; }); }
__device__ inline double sum(double v) { return all(v, [](double a, double b) { return a + b; }); }
__device__ inline double max(double v) { return all(v, [](double a, double b) { return fmax(a, b); }); }
__device__ inline float row_sum(float v) { return row_all(v, [](float a, float b) { return a + b; }); }


// Rank counting for a top-k selection by several waves.  logit[0 .. E) and rank[0 .. E) live in
// LDS, rank zeroed.  The calling wave adds to rank[e] the number of logits e2 = first,
// first + stride, ... that come before logit e in the order (larger first, lower index first
// among equals); with every e2 covered by some wave, rank[] becomes the position of each logit in
// that strict order.  Lane l keeps logits l, l + 64, ... (NR of them, NR >= ceil(E / 64)) in
// registers; the logits e2 are broadcast reads, kBatch in flight, compared without branches
// (every comparison leaves a mask in scalar registers: a smaller batch where those are scarce).
template <int NR, int kBatch = 8>
__device__ inline void count_ranks(const double *logit, int32_t *rank, int E, int lane, int first, int stride)
{
    double mine[NR];
    int part[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const int e = lane + 64 * i;
        mine[i] = logit[e < E ? e : E - 1];
        part[i] = 0;
    }
    for (int e2 = first; e2 < E; e2 += kBatch * stride) {
        double v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int idx = e2 + j * stride;
            v[j] = logit[idx < E ? idx : E - 1];
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int idx = e2 + j * stride;
            const int live = idx < E ? 1 : 0;
#pragma unroll
            for (int i = 0; i < NR; ++i)
                part[i] += live & ((int)(v[j] > mine[i]) | ((int)(v[j] == mine[i]) & (int)(idx < lane + 64 * i)));
        }
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const int e = lane + 64 * i;
        if (e < E && part[i] != 0) atomicAdd(&rank[e], part[i]);
    }
}
__device__ inline void count_ranks(const double *logit, int32_t *rank, int E, int lane, int first, int stride)
{
    if (E <= 64) count_ranks<1>(logit, rank, E, lane, first, stride);
    else if (E <= 128) count_ranks<2>(logit, rank, E, lane, first, stride);
    else count_ranks<4>(logit, rank, E, lane, first, stride);
}

}  // namespace wave
}  // namespace moespeq
