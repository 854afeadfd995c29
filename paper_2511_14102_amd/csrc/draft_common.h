// Shared pieces of the two draft-pass kernel files (gfx950): the arithmetic helpers of the int4
// path (code unpacking into exact bf16 integers, MFMA wrapper, scale / zero entries), agent-scope
// 16-byte accesses of the router exchange, and the kernels' argument block.
//
// Arithmetic (paper section 4.1.3: 4-bit weights in groups along the input dimension).
// W = (q - z) * s, so for one output row and one group G of inputs
//     sum_{c in G} W[c] v[c] = s * ( sum_c (128 + q[c]) v[c]  -  (z + 128) * sum_c v[c] ).
// 0x4300 is bf16 128.0 with a zero mantissa, so or-ing a code into mantissa bits 0-3 gives the
// bf16 value 128 + q exactly: unpacking is one shift and one and-or per pair of codes.  The
// products and sums are then done by the matrix cores (16x16x32 bf16 MFMA, fp32 accumulation):
// the unpacked codes of 16 weight rows are the B operand, the activations of up to 16 tokens the
// A operand.  Scale, zero and the 128 offset are applied once per group on the accumulators.
#pragma once
#include <type_traits>
#include "plan.h"
#include "wave.h"

namespace moespeq {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
// The router result is published in kReplicas copies; workgroup b polls copy b % kReplicas, so
// that the polls of hundreds of workgroups do not all land on one address.
constexpr int kReplicas = kDraftSlotReplicas;
constexpr int kTicketGroups = 16;
// Up to this many experts the wave that polled a token's logits also selects its top-k by itself;
// beyond, all waves share the ranking (two more barriers, which cost more than they save on few
// experts: measured 1 us on 16 experts).
constexpr int kLoneWaveTopk = 32;
constexpr uint32_t kMagic = 0x43004300u;      // bf16 pair (128, 128)

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Unpack constants.  Both are made opaque to the compiler (one in a scalar, one in a vector
// register) so that (a & mask) | magic has no literal operand and is selected as the single
// instruction v_and_or_b32.  It must be the compiler's own instruction, not inline assembly:
// the hazard recogniser does not see inline assembly as a VALU write, and an MFMA that read
// such a result directly got a stale operand (wrong results on the GPU).
struct UnpackConsts { uint32_t mask, magic; };
__device__ inline UnpackConsts unpack_consts() {
    UnpackConsts k = {0x000F000Fu, kMagic};
    asm volatile("" : "+s"(k.mask));
    asm volatile("" : "+v"(k.magic));
    return k;
}

// The 8 codes of one 32-bit word as 8 bf16 values 128 + code, in code order (an MFMA operand)
__device__ inline bf16x8 unpack8(uint32_t w, UnpackConsts k) {
    u32x4 r;
    r.x = (w & k.mask) | k.magic;
    r.y = ((w >> 4) & k.mask) | k.magic;
    r.z = ((w >> 8) & k.mask) | k.magic;
    r.w = ((w >> 12) & k.mask) | k.magic;
    return __builtin_bit_cast(bf16x8, r);
}

__device__ inline f32x4 mfma(u32x4 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), b, c, 0, 0, 0);
}

// One 16-byte load at agent scope (served by the device's coherence point, not a stale cache line)
__device__ inline u32x4 load16_agent(const void *p) {
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}

__device__ inline void store16_agent(void *p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

// 1 KiB of device memory (16 bytes per lane, at the lane's address g) straight into LDS at byte
// offset lds_base (wave-uniform) + 16 * lane.  Issued as assembly on purpose: the compiler then
// does not know of the transfer and adds no waits of its own for it (it would wait for ALL vector
// memory operations before every barrier and every LDS read that follows); the caller orders the
// use of the data behind the arrival of a later load of the same wave (vector memory operations
// complete in order).
__device__ inline void load16_to_lds(const void *g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(g) : "memory");
}

struct FusedArgs {
    const uint16_t *wr;         // [E,H] bf16
    const float *bias;          // [E] or null
    const char *q;              // int4 codes blobs
    const char *sz;             // scale/zero blobs
    size_t stride_q, stride_sz;
    unsigned long long *slots;  // kReplicas x [T,E] x {logit bits, tag}; idle: tag = 0
    size_t replica_stride;      // in 8-byte units
    uint32_t *tickets;          // kTicketGroups + 1 counters; idle: 0
    uint32_t *status;           // set to 1 when a wait for the router result ran out of polls
    uint32_t spin_limit;        // polls of the router result before a workgroup gives up
    float *y;                   // [T,H] out, accumulated with atomics
    int32_t *ids_out;           // [T,k]
    float *conf_out;            // [T,k] or null
    Plan *plan;                 // filled for the shared-expert kernels when S > 0
    const char *shared;         // bf16 shared expert blobs
    size_t shared_stride;
    int T, H, E, I, k, g, S, renorm;
};

// Scale and zero of the four row blocks d of one (group, lane row): the asymmetric format keeps
// a 4-byte {s, z} entry per d, the symmetric one (z = 8) only the four fp16 scales.
template <bool SYM> struct GroupParams;
template <> struct GroupParams<false> {
    uint32_t w[4];
    // entry d; d may differ from lane to lane, so the choice is made with bit masks (a chain of
    // conditional expressions on a lane-varying d was compiled into divergent branches)
    __device__ uint32_t entry(int d) const {
        const uint32_t m1 = 0u - (uint32_t)(d & 1), m2 = 0u - (uint32_t)((d >> 1) & 1);
        const uint32_t lo = (w[1] & m1) | (w[0] & ~m1), hi = (w[3] & m1) | (w[2] & ~m1);
        return (hi & m2) | (lo & ~m2);
    }
    __device__ float scale(int d) const { return (float)__builtin_bit_cast(_Float16, (uint16_t)(entry(d) & 0xffff)); }
    __device__ float zero128(int d) const {                   // z + 128
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(entry(d) >> 16)) + 128.f;
    }
};
template <> struct GroupParams<true> {
    uint32_t w[2];
    __device__ float scale(int d) const {
        const uint32_t m2 = 0u - (uint32_t)((d >> 1) & 1);
        const uint32_t e = (w[1] & m2) | (w[0] & ~m2);
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(e >> (16 * (d & 1))));
    }
    __device__ float zero128(int) const { return 136.f; }
};


// Launch with `lds` bytes of dynamic LDS; beyond 48 KiB the limit has to be raised once per kernel.
template <typename K>
void launch_with_lds(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, const uint16_t *x,
                     const FusedArgs &a)
{
    static size_t raised = 0;                    // per instantiation
    if (lds > 48 * 1024 && lds > raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        raised = lds;
    }
    launch(kernel, grid, block, lds, st, x, a);
}

// workgroups of `kernel` (block threads, lds bytes of dynamic LDS) one compute unit holds at once
template <typename K>
int resident_per_cu(K kernel, int threads, size_t lds)
{
    if (lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds) != hipSuccess) return 0;
    return n;
}

inline FusedArgs fused_args(const Shape &s, const DraftFusedArgs &d)
{
    FusedArgs a;
    a.wr = (const uint16_t *)d.wr; a.bias = d.bias;
    a.q = (const char *)d.q; a.sz = (const char *)d.sz; a.stride_q = d.stride_q; a.stride_sz = d.stride_sz;
    a.slots = d.slots; a.replica_stride = d.replica_stride; a.tickets = d.tickets; a.y = d.y;
    a.status = d.status; a.spin_limit = d.spin_limit;
    a.ids_out = d.ids_out; a.conf_out = d.conf_out; a.plan = d.plan;
    a.shared = (const char *)d.shared; a.shared_stride = d.shared_stride;
    a.T = s.T; a.H = s.H; a.E = s.E; a.I = s.I; a.k = s.k; a.g = s.g; a.S = s.S; a.renorm = s.renorm;
    return a;
}

}  // namespace

}  // namespace moespeq
