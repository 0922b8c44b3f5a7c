// Scatter of the correct items' gradient rows, shared by the matrix-core kernels and the per-position path.
#pragma once
#include "cce_device.hpp"
#include "cce_kernels.hpp"

namespace cce {

// Position row of compacted index x (identity when there is no mask).
__device__ __forceinline__ int64_t pos_row(const TileArgs &a, int64_t x) { return a.idx ? (int64_t)a.idx[x] : x; }

// dE of the correct items: dE[tgt_i] += coef_i * H_i.  Targets follow a power law, so plain atomics would serialise
// on a few hot rows (an atomic on one address completes every ~25 ns).  A block sorts 256 (target, position) pairs in
// LDS; every wavefront then walks 64 consecutive sorted pairs with lane = column, sums runs of equal targets in
// registers and issues one row of atomics per run.  These blocks ride at the head of another launch (the dE pass of the
// matrix-core path, the second index pass of the per-position path), so that their latency (sort, dependent gathers)
// hides under that launch's own work.  Where the scatter is a launch of its own a block sorts 1024 pairs: longer runs
// of equal targets, fewer rows of atomics (largest workload: 60 k instead of 78 k).
constexpr int kPosChunk = 256;        // pairs per block riding in another launch
constexpr int kPosChunkApart = 1024;  // pairs per block of the stand-alone scatter kernels

template <int D, int CHUNK = kPosChunk>
__device__ __forceinline__ void pos_scatter_block(const TileArgs &a, int64_t chunk, uint64_t *keys)
{
    constexpr int CPL = D / 64;         // columns per lane
    constexpr int kPosBatch = 16;        // rows in flight per wavefront
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t base = chunk * CHUNK;
    if (base >= n_pos) return;
    const bool sorter = tid < CHUNK;  // blocks of more threads than pairs: the rest only keep the barriers company
    if (sorter) {
        uint64_t key = ~0ull;  // padding sorts last
        if (base + tid < n_pos) {
            const int64_t row = pos_row(a, base + tid);
            if (!a.pos_mask || a.pos_mask[row] != 0) {  // ids of padded positions are never read
                const int32_t ti = a.tgt[row];
                if (!a.validate || (ti >= 0 && (int64_t)ti < a.V)) key = ((uint64_t)(uint32_t)ti << 32) | (uint32_t)row;
            }
        }
        keys[tid] = key;
    }
    __syncthreads();
    for (int k = 2; k <= CHUNK; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int partner = tid ^ j;
            if (sorter && partner > tid) {
                const uint64_t ka = keys[tid], kb = keys[partner];
                const bool up = ((tid & k) == 0);
                if ((ka > kb) == up) {
                    keys[tid] = kb;
                    keys[partner] = ka;
                }
            }
            __syncthreads();
        }
    }

    if (!sorter) return;  // no barrier below this point
    float accv[CPL];
#pragma unroll
    for (int t = 0; t < CPL; ++t) accv[t] = 0.f;
    uint32_t cur = 0xffffffffu;
    auto flush = [&]() {
        if (cur != 0xffffffffu) {
#pragma unroll
            for (int t = 0; t < CPL; ++t) {
                unsafeAtomicAdd(a.dE + (int64_t)cur * D + t * 64 + lane, accv[t]);  // an instruction covers 64 consecutive floats
                accv[t] = 0.f;
            }
        }
    };
    // lane l holds pair l of the wavefront's 64 sorted pairs and its coefficient; the walk broadcasts them lane by lane
    const uint64_t my_key = keys[wave * 64 + lane];
    const uint32_t my_id = (uint32_t)(my_key >> 32), my_row = (uint32_t)my_key;
    const float my_cf = (my_id != 0xffffffffu) ? a.coef[my_row] * ((a.g_separate && a.g) ? a.g[my_row] : 1.f) : 0.f;
    for (int b = 0; b < 64; b += kPosBatch) {
        uint32_t id[kPosBatch];
        float hv[kPosBatch][CPL];
#pragma unroll
        for (int u = 0; u < kPosBatch; ++u) {
            id[u] = __builtin_amdgcn_readlane(my_id, b + u);
            const uint32_t row = __builtin_amdgcn_readlane(my_row, b + u);
#pragma unroll
            for (int t = 0; t < CPL; ++t) hv[u][t] = 0.f;
            if (id[u] != 0xffffffffu) {
#pragma unroll
                for (int t = 0; t < CPL; ++t) hv[u][t] = load1(a.H + (int64_t)row * D + t * 64 + lane);
            }
        }
#pragma unroll
        for (int u = 0; u < kPosBatch; ++u) {
            if (id[u] != cur) {
                flush();
                cur = id[u];
            }
            const float cf = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_cf), b + u));
#pragma unroll
            for (int t = 0; t < CPL; ++t) accv[t] = fmaf(cf, hv[u][t], accv[t]);
        }
    }
    flush();
}

}  // namespace cce
