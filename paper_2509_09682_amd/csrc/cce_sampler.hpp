// Negative sampling inside the loss kernels: item ids as a pure function of (seed, stream, position, draw number).
//
// The paper samples the negatives of a step on the host (global uniform, or by popularity through a multinomial over
// the catalogue; Sec. 5, "Comparison Sampling Strategies") and names the stored index matrix as the memory overhead
// of CCE- (Sec. 5, "What is better").  With a counter-based generator the forward pass, the backward pass and the
// index build regenerate the same ids instead of reading them, so the matrix never exists.
//
//   generator : Philox4x32-10 (Salmon et al., SC'11); key = the two halves of the seed,
//               counter = (q, position low, position high, stream)
//   slot s of a position is draw j = s + 1
//   uniform   : q = j >> 2, r = word j & 3, id = floor(r V / 2^32)
//   alias     : q = j >> 1, (r0, r1) = words 2(j & 1), 2(j & 1) + 1, column c = floor(r0 V / 2^32),
//               id = r1 < thresh[c] ? c : alias[c]           (Walker / Vose table supplied by the caller)
//   shared negatives are the draws of position 0.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cce {

struct Sampler {
    uint32_t kind;            // 0 = off (ids are read from memory), else cce_sampler_kind
    uint32_t k0, k1, stream;
    uint32_t V;
    const uint32_t *thresh;   // alias method: [V] keep thresholds in units of 2^-32
    const int32_t *alias;     // alias method: [V]
};

enum { kSamplerUniform = 1, kSamplerAlias = 2 };

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                              uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(M0, c0), l0 = M0 * c0;
        const uint32_t h1 = __umulhi(M1, c2), l1 = M1 * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Ids of the four consecutive draws j = 4 q4 .. 4 q4 + 3 of a position (both laws).
__device__ __forceinline__ void sample4(const Sampler &s, uint64_t pos, uint32_t q4, int32_t (&id)[4])
{
    const uint32_t p_lo = (uint32_t)pos, p_hi = (uint32_t)(pos >> 32);
    uint32_t w[4];
    if (s.kind == kSamplerUniform) {
        philox4x32_10(q4, p_lo, p_hi, s.stream, s.k0, s.k1, w);
#pragma unroll
        for (int t = 0; t < 4; ++t) id[t] = (int32_t)__umulhi(w[t], s.V);
    } else {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            philox4x32_10(2 * q4 + half, p_lo, p_hi, s.stream, s.k0, s.k1, w);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t col = __umulhi(w[2 * t], s.V);
                id[2 * half + t] = (w[2 * t + 1] < s.thresh[col]) ? (int32_t)col : s.alias[col];
            }
        }
    }
}

// Id of a single draw.
__device__ __forceinline__ int32_t sample1(const Sampler &s, uint64_t pos, uint32_t j)
{
    const uint32_t p_lo = (uint32_t)pos, p_hi = (uint32_t)(pos >> 32);
    uint32_t w[4];
    if (s.kind == kSamplerUniform) {
        philox4x32_10(j >> 2, p_lo, p_hi, s.stream, s.k0, s.k1, w);
        const uint32_t r = (j & 2) ? ((j & 1) ? w[3] : w[2]) : ((j & 1) ? w[1] : w[0]);
        return (int32_t)__umulhi(r, s.V);
    }
    philox4x32_10(j >> 1, p_lo, p_hi, s.stream, s.k0, s.k1, w);
    const uint32_t r0 = (j & 1) ? w[2] : w[0], r1 = (j & 1) ? w[3] : w[1];
    const uint32_t col = __umulhi(r0, s.V);
    return (r1 < s.thresh[col]) ? (int32_t)col : s.alias[col];
}

}  // namespace cce
