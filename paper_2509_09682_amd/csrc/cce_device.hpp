// Shared device-side helpers and the kernel parameter block of the CCE- library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cce_neg.h"
#include "cce_sampler.hpp"

namespace cce {

// Everything a kernel needs, passed by value at launch.
struct Params {
    const void *H;          // [N,d] in_dtype
    const void *E;          // [V,d] in_dtype
    const int32_t *tgt;     // [N]
    const int32_t *neg;     // [K] | [N,K] | nullptr
    const uint8_t *mask;    // [N] | nullptr
    const float *lse_in;    // [N] (backward)
    const float *g;         // [N] | nullptr (backward)
    float *loss;            // [N] (forward)
    float *lse;             // [N] (forward)
    void *dH;               // [N,d] (backward)
    float *dE;              // [V,d] (backward)
    int32_t *status;        // index status word in the workspace header
    int64_t N, V;
    int32_t d, K;
    int32_t neg_mode, collide, validate, dH_bf16;
    // backward of the row-gather family when dE of the negatives is produced by the inverted-index pass instead:
    int32_t skip_neg_dE;    // 1: no dE atomics for negatives
    int32_t skip_pos_dE;    // 1: no dE atomics for the correct item either (the aggregated scatter adds it)
    float *coef;            // [N] out: g_i (p+_i - 1), coefficient of the correct item (nullable); the fused forward pass
                            // files p+_i - 1 there, short of the upstream gradient
    float *U;               // [N,d] fp32, fused forward pass: sum_j softmax_ij E_cij - E_tgt_i (Eq. 6 left with grad LSE = 1);
                            // the backward call scales it by grad_loss
    Sampler smp;            // per-position mode, kind != 0: the negatives are drawn in the kernel, neg is not read
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x)
{
    uint32_t b = __float_as_uint(x);
    return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// Load 8 consecutive elements (16-byte aligned for bf16, 32-byte for fp32) and widen to float.
__device__ __forceinline__ void load8(const float *p, float (&v)[8])
{
    const float4 a = reinterpret_cast<const float4 *>(p)[0];
    const float4 b = reinterpret_cast<const float4 *>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const uint16_t *p, float (&v)[8])
{
    const uint4 r = *reinterpret_cast<const uint4 *>(p);
    v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x);
    v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
    v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z);
    v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
}
// A row chunk of 8 elements as it comes from memory; bf16 rows stay packed (4 registers) until they are used, so that
// twice as many rows can be in flight per wavefront as with widened copies.
template <typename T> struct RawChunk;
template <> struct RawChunk<uint16_t> {
    uint4 v;
    static constexpr int kInFlight = 8;
    __device__ __forceinline__ void load(const uint16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void clear() { v = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void widen(float (&h)[8]) const
    {
        h[0] = bf16_lo(v.x); h[1] = bf16_hi(v.x);
        h[2] = bf16_lo(v.y); h[3] = bf16_hi(v.y);
        h[4] = bf16_lo(v.z); h[5] = bf16_hi(v.z);
        h[6] = bf16_lo(v.w); h[7] = bf16_hi(v.w);
    }
};
template <> struct RawChunk<float> {
    float4 a, b;
    static constexpr int kInFlight = 4;
    __device__ __forceinline__ void load(const float *p)
    {
        a = reinterpret_cast<const float4 *>(p)[0];
        b = reinterpret_cast<const float4 *>(p)[1];
    }
    __device__ __forceinline__ void clear() { a = b = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void widen(float (&h)[8]) const
    {
        h[0] = a.x; h[1] = a.y; h[2] = a.z; h[3] = a.w;
        h[4] = b.x; h[5] = b.y; h[6] = b.z; h[7] = b.w;
    }
};

// Streaming accesses (data used once): loads and stores marked non-temporal leave the L2 lines they touch first in
// line for eviction, so that a small operand that IS reused (the hidden states in the item pass) stays resident.
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load(const float4 *p)
{
    const f32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store(float4 *p, float4 v)
{
    f32x4_nt w;
    w.x = v.x; w.y = v.y; w.z = v.z; w.w = v.w;
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4_nt *>(p));
}
__device__ __forceinline__ int32_t stream_load(const int32_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void stream_load8(const float *p, float (&v)[8])
{
    const float4 a = stream_load(reinterpret_cast<const float4 *>(p)), b = stream_load(reinterpret_cast<const float4 *>(p) + 1);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void stream_load8(const uint16_t *p, float (&v)[8])
{
    const u32x4_nt r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(p));
    v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x);
    v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
    v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z);
    v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
}

__device__ __forceinline__ float load1(const float *p) { return *p; }
__device__ __forceinline__ float load1(const uint16_t *p) { return __uint_as_float(static_cast<uint32_t>(*p) << 16); }

// exp(x) and log(x) through the base-2 hardware units.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * kLn2; }

// Merge two (max, sum-of-exp) pairs of an online softmax; either may be the empty pair (-inf, 0).
__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2)
{
    const float M = fmaxf(m, m2);
    if (M == -INFINITY) { s = 0.f; return; }
    s = s * fast_exp(m - M) + s2 * fast_exp(m2 - M);
    m = M;
}

}  // namespace cce
