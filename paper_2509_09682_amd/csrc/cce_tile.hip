// Matrix-core family, what does not depend on the hidden size: the preparation kernel and the dispatch to the
// per-hidden-size files (cce_tile_d64.hip, cce_tile_d128.hip, cce_tile_d256.hip; kernel template in cce_tile_body.hpp).
#include "cce_device.hpp"
#include "cce_kernels.hpp"
#include "cce_tile_shared.hpp"

namespace cce {
namespace {

// ---------------------------------------------------------------------------------------------------------------------
// Preparation: compaction of the valid positions, zero rows for the padded ones, and the multiplicity c_i of each
// position's target among the shared negatives (through a hash table of the negatives built in LDS by every block).
constexpr int kPrepThreads = 1024;
constexpr int kTgtSlots = 2048;  // LDS hash table of the block's own targets; load factor <= 1/2, so probing always ends

__device__ __forceinline__ uint32_t hash_id(int32_t id, int slots) { return (((uint32_t)id * 2654435761u) >> 15) & (uint32_t)(slots - 1); }

// Number of non-zero bytes in a 32-bit word.
__device__ __forceinline__ int nonzero_bytes(uint32_t w)
{
    return __popc((w | ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u);
}

// Every block handles 1024 consecutive positions.  The slot of a valid position in the compacted list is its rank
// among all valid positions, so the list keeps the original order and needs no atomics: a block finds the number of
// valid positions in front of it by counting the mask bytes of that prefix itself (N bytes at most, from L2).
__global__ __launch_bounds__(kPrepThreads) void prep_kernel(PrepArgs p)
{
    __shared__ int32_t hkey[kTgtSlots];
    __shared__ int32_t hcnt[kTgtSlots];
    __shared__ int32_t wave_count[kPrepThreads / 64];
    __shared__ int32_t wave_prefix[kPrepThreads / 64];
    __shared__ int32_t block_base;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * kPrepThreads;
    const int64_t i = i0 + tid;
    bool valid = false;
    int32_t ti = 0;
    if (i < p.N) {
        valid = (p.mask == nullptr) || (p.mask[i] != 0);
        if (valid) {
            ti = p.tgt[i];
            if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) {
                valid = false;
                atomicOr(p.header + kHdrStatus, 1);
            }
        }
    }

    if (p.idx) {
        // ---- valid positions in front of this block
        int32_t before = 0;
        if (p.validate) {  // validity depends on the target too: walk positions one by one
            for (int64_t j = tid; j < i0; j += kPrepThreads) {
                const bool m = (p.mask == nullptr) || (p.mask[j] != 0);
                if (m) {
                    const int32_t t = p.tgt[j];
                    before += (t >= 0 && (int64_t)t < p.V) ? 1 : 0;
                }
            }
        } else if (p.mask) {  // i0 is a multiple of 1024, the mask is 16-byte aligned
            const uint4 *m16 = reinterpret_cast<const uint4 *>(p.mask);
            const int64_t n16 = i0 / 16;
            int64_t c = tid;
            for (; c + 3 * kPrepThreads < n16; c += 4 * kPrepThreads) {  // four loads in flight: the walk is a chain of latencies
                const uint4 v0 = m16[c], v1 = m16[c + kPrepThreads], v2 = m16[c + 2 * kPrepThreads], v3 = m16[c + 3 * kPrepThreads];
                before += nonzero_bytes(v0.x) + nonzero_bytes(v0.y) + nonzero_bytes(v0.z) + nonzero_bytes(v0.w);
                before += nonzero_bytes(v1.x) + nonzero_bytes(v1.y) + nonzero_bytes(v1.z) + nonzero_bytes(v1.w);
                before += nonzero_bytes(v2.x) + nonzero_bytes(v2.y) + nonzero_bytes(v2.z) + nonzero_bytes(v2.w);
                before += nonzero_bytes(v3.x) + nonzero_bytes(v3.y) + nonzero_bytes(v3.z) + nonzero_bytes(v3.w);
            }
            for (; c < n16; c += kPrepThreads) {
                const uint4 v = m16[c];
                before += nonzero_bytes(v.x) + nonzero_bytes(v.y) + nonzero_bytes(v.z) + nonzero_bytes(v.w);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) before += __shfl_xor(before, off, 64);
        const uint64_t ballot = __ballot(valid);
        const int rank_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
        if (lane == 0) {
            wave_count[wave] = __popcll(ballot);
            wave_prefix[wave] = before;  // partial sum of the prefix count held by this wavefront
        }
        __syncthreads();
        if (tid == 0) {
            int32_t base = 0, run = 0;
            for (int w = 0; w < kPrepThreads / 64; ++w) base += wave_prefix[w];
            for (int w = 0; w < kPrepThreads / 64; ++w) {
                const int32_t c = wave_count[w];
                wave_count[w] = run;
                run += c;
            }
            block_base = base;
            if (blockIdx.x == gridDim.x - 1) p.header[kHdrNValid] = base + run;  // the last block knows the total
        }
        __syncthreads();
        if (valid) p.idx[block_base + wave_count[wave] + rank_in_wave] = (int32_t)i;
    }

    // ---- rows of padded positions are zero
    if (i < p.N && !valid) {
        if (p.loss) p.loss[i] = 0.f;
        if (p.lse) p.lse[i] = 0.f;
    }

    // ---- multiplicity of each target among the shared negatives: the block's targets go into an LDS hash table,
    //      the K negatives are streamed past it, every hit bumps the count of its slot
    if (p.cnt) {
        for (int s = tid; s < kTgtSlots; s += kPrepThreads) {
            hkey[s] = -1;
            hcnt[s] = 0;
        }
        __syncthreads();
        int my_slot = -1;
        if (valid) {
            uint32_t h = hash_id(ti, kTgtSlots);
            for (int probe = 0; probe < kTgtSlots; ++probe) {
                const int32_t prev = atomicCAS(&hkey[h], -1, ti);
                if (prev == -1 || prev == ti) {
                    my_slot = (int)h;
                    break;
                }
                h = (h + 1) & (kTgtSlots - 1);
            }
        }
        __syncthreads();
        auto count_hit = [&](int32_t id) {
            if (id < 0) return;  // flagged by the range check below; never equal to a valid target
            uint32_t h = hash_id(id, kTgtSlots);
            for (int probe = 0; probe < kTgtSlots; ++probe) {
                const int32_t key = hkey[h];
                if (key == id) {
                    atomicAdd(&hcnt[h], 1);
                    break;
                }
                if (key == -1) break;
                h = (h + 1) & (kTgtSlots - 1);
            }
        };
        int64_t k = tid;
        for (; k + 3 * kPrepThreads < p.K; k += 4 * kPrepThreads) {  // ids of four rounds fetched together
            const int32_t id0 = p.neg[k], id1 = p.neg[k + kPrepThreads], id2 = p.neg[k + 2 * kPrepThreads], id3 = p.neg[k + 3 * kPrepThreads];
            count_hit(id0);
            count_hit(id1);
            count_hit(id2);
            count_hit(id3);
        }
        for (; k < p.K; k += kPrepThreads) count_hit(p.neg[k]);
        __syncthreads();
        if (valid) p.cnt[i] = hcnt[my_slot];
    }

    // ---- range check of the shared negatives (once, by block 0)
    if (p.validate && p.neg && blockIdx.x == 0) {
        bool bad = false;
        for (int64_t k = tid; k < p.K; k += kPrepThreads) {
            const int32_t id = p.neg[k];
            bad |= (id < 0 || (int64_t)id >= p.V);
        }
        if (bad) atomicOr(p.header + kHdrStatus, 1);
    }
}

}  // namespace

hipError_t launch_tile_d64(int pass, const TileArgs &a, hipStream_t stream);
hipError_t launch_tile_d128(int pass, const TileArgs &a, hipStream_t stream);
hipError_t launch_tile_d256(int pass, const TileArgs &a, hipStream_t stream);
hipError_t launch_tile_backward_d64(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream);
hipError_t launch_tile_backward_d128(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream);
hipError_t launch_pos_scatter_d64(const TileArgs &a, hipStream_t stream);
hipError_t launch_pos_scatter_d128(const TileArgs &a, hipStream_t stream);
hipError_t launch_pos_scatter_d256(const TileArgs &a, hipStream_t stream);
hipError_t launch_dh_scale_d64(const TileArgs &a, bool file_g, hipStream_t stream);
hipError_t launch_dh_scale_d128(const TileArgs &a, bool file_g, hipStream_t stream);
hipError_t launch_dh_scale_d256(const TileArgs &a, bool file_g, hipStream_t stream);

bool tile_supports_d(int d) { return d == 64 || d == 128 || d == 256; }
size_t tile_tail_partial_bytes(int64_t N, int d) { return (d > 128 && N > kTailRows) ? (size_t)kTailRows * d * 4 : 0; }

hipError_t launch_pos_scatter(const TileArgs &a, hipStream_t stream)
{
    switch (a.d) {
    case 64: return launch_pos_scatter_d64(a, stream);
    case 128: return launch_pos_scatter_d128(a, stream);
    case 256: return launch_pos_scatter_d256(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_dh_scale(const TileArgs &a, bool file_g, hipStream_t stream)
{
    switch (a.d) {
    case 64: return launch_dh_scale_d64(a, file_g, stream);
    case 128: return launch_dh_scale_d128(a, file_g, stream);
    case 256: return launch_dh_scale_d256(a, file_g, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_prep(const PrepArgs &p, hipStream_t stream)
{
    if (p.N == 0) return hipSuccess;
    ProfScope prof(PROF_PREP, stream);
    hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((p.N + kPrepThreads - 1) / kPrepThreads)), dim3(kPrepThreads), 0,
                       stream, p);
    return hipGetLastError();
}

bool tile_backward_fusable(int d) { return d == 64 || d == 128; }

hipError_t launch_tile_backward(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream)
{
    if (a_dh.N == 0) return hipSuccess;
    switch (a_dh.d) {
    case 64: return launch_tile_backward_d64(a_dh, a_de, stream);
    case 128: return launch_tile_backward_d128(a_dh, a_de, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_tile(int pass, const TileArgs &a, hipStream_t stream)
{
    if (a.N == 0) return hipSuccess;
    switch (a.d) {
    case 64: return launch_tile_d64(pass, a, stream);
    case 128: return launch_tile_d128(pass, a, stream);
    case 256: return launch_tile_d256(pass, a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace cce
