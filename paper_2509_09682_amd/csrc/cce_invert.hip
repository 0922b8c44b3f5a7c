// dE of per-position negatives through an inverted index (item -> the (position, slot) pairs that sampled it).
//
// Alg. 2 updates the classifier gradient with one indexed row add per (position, candidate) pair.  With N*K pairs
// spread over a large table that is N*K*d floating-point atomics, and this chip retires scattered fp32 atomics at about
// 1.3 TB/s of payload against 7 TB/s for plain stores.  The same sum can be taken item by item: count the pairs of
// every item, turn the counts into offsets, file each pair under its item (a counting sort with integer atomics on a
// V-word table), then let one lane group per item recompute its few scores against hidden states that sit in L2 and
// add the finished row to dE once, without atomics.  Table rows are read once and written once; no score is stored.
// The correct items (power-law hot rows) are not part of the index: the aggregated scatter adds them.
#include "cce_device.hpp"
#include "cce_kernels.hpp"
#include "cce_scatter.hpp"

namespace cce {
namespace {

constexpr int kThreads = 256;

// One thread per (position, slot) pair of a valid position whose negative takes part.
__device__ __forceinline__ bool pair_live(const InvertArgs &a, int64_t pair, int32_t &id)
{
    const int64_t i = pair / a.K;
    if (a.mask && a.mask[i] == 0) return false;
    id = a.smp.kind ? sample1(a.smp, (uint64_t)i, (uint32_t)(pair - i * a.K) + 1u) : a.neg[pair];
    const int32_t ti = a.tgt[i];
    if (a.validate && (ti < 0 || (int64_t)ti >= a.V || id < 0 || (int64_t)id >= a.V)) return false;  // flagged elsewhere
    return !(a.collide && id == ti);
}

// ---- exclusive scan of an int array in two launches: block-local scan + block totals, then every block adds the
//      totals of the blocks in front of it (read directly: n/4096 values at most)
constexpr int kScanThreads = 1024;
constexpr int kScanItems = 4;
constexpr int kScanChunk = kScanThreads * kScanItems;

__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t *lds, int32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    __syncthreads();  // lds may still be read from a previous call
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int w = 0; w < kScanThreads / 64; ++w) {
            const int32_t c = lds[w];
            lds[w] = run;
            run += c;
        }
        lds[kScanThreads / 64] = run;
    }
    __syncthreads();
    total = lds[kScanThreads / 64];
    return incl - v + lds[wave];
}

__global__ __launch_bounds__(kScanThreads) void scan_local_kernel(int32_t *data, int64_t n, int32_t *block_sums)
{
    __shared__ int32_t lds[kScanThreads / 64 + 1];
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int32_t v[kScanItems], sum = 0;
#pragma unroll
    for (int t = 0; t < kScanItems; ++t) {
        v[t] = (base + t < n) ? data[base + t] : 0;
        sum += v[t];
    }
    int32_t total;
    int32_t run = block_exclusive_scan(sum, lds, total);
#pragma unroll
    for (int t = 0; t < kScanItems; ++t) {
        if (base + t < n) data[base + t] = run;
        run += v[t];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void scan_add_kernel(int32_t *data, int64_t n, const int32_t *block_sums)
{
    __shared__ int32_t lds[kScanThreads / 64 + 1];
    int32_t part = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += kScanThreads) part += block_sums[b];
    int32_t total;
    (void)block_exclusive_scan(part, lds, total);
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
#pragma unroll
    for (int t = 0; t < kScanItems; ++t)
        if (base + t < n) data[base + t] += total;
}

hipError_t launch_scan(int32_t *data, int64_t n, int32_t *block_sums, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((n + kScanChunk - 1) / kScanChunk);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(scan_local_kernel, dim3(blocks), dim3(kScanThreads), 0, stream, data, n, block_sums);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scan_add_kernel, dim3(blocks), dim3(kScanThreads), 0, stream, data, n, block_sums);
    return hipGetLastError();
}

// ---- fallback index build for huge catalogues: integer atomics on the V-word table (scattered atomics are slow:
//      about 27 G/s for the count, 10 G/s for the returning ones of the fill)
__global__ __launch_bounds__(kThreads) void count_kernel(InvertArgs a)
{
    const int64_t pair = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (pair >= a.N * a.K) return;
    int32_t id;
    if (pair_live(a, pair, id)) atomicAdd(a.cursor + id, 1);
}

// File every live pair under its item.  Afterwards cursor[v] is the END of item v's segment; it starts where the
// segment of v-1 ends.
__global__ __launch_bounds__(kThreads) void fill_kernel(InvertArgs a)
{
    const int64_t pair = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (pair >= a.N * a.K) return;
    int32_t id;
    if (pair_live(a, pair, id)) {
        const int32_t slot = atomicAdd(a.cursor + id, 1);
        a.pairs[slot] = (int32_t)(pair / a.K);  // only the position is needed downstream
    }
}

// ---- index build by two-level counting sort without global atomics.
//  Level 1 partitions the pairs into buckets of kBucketIds consecutive item ids: every block histograms its chunk of
//  pairs in LDS, the (bucket, block) counts are scanned bucket-major, and the block scatters (id, position) into its
//  reserved ranges.  Level 2 gives each bucket to one block, which counting-sorts it by id inside LDS and writes the
//  positions item by item together with the end offset of every item.
constexpr int kBucketShift = 11;
constexpr int kBucketIds = 1 << kBucketShift;  // LDS histogram of level 2: 8 KiB
constexpr int kMaxBuckets = 2048;               // LDS histogram of level 1: 8 KiB
constexpr int kChunkPairs = 8192;               // pairs per chunk in level 1; a block takes chunks blockIdx.x, + gridDim.x, ...
constexpr int kMaxPartBlocks = 4096;            // blocks of level 1: bounds the (bucket, block) histogram at 32 MiB
// The index is built and used up in SLICES of the item-id range, so that its memory is bounded by a pair budget B instead
// of growing with N * K: every slice is a run of consecutive buckets that holds at most B pairs, gets filed into the same
// B-entry arrays, and is consumed by the item pass before the next one is filed.  Every table row is still read and
// written once; a further slice costs one more reading of the ids (4 bytes per pair) and four launches.
//   B = max(2^22, N K / 8) pairs;  slices = 1 if N K <= B, else ceil(N K / (7/8 B)): the pairs of the ordinary buckets
//   are cut at the quantiles j / slices of their running count, so a slice holds at most N K / slices + (one bucket)
//   <= 7/8 B + 1/8 B pairs, PROVIDED no bucket holds more than B / 8 pairs.  Buckets beyond that (2048 consecutive ids
//   drawing more than half a million pairs, an eighth of everything: a popularity law far more skewed than any workload
//   here) stay out of the index: their pairs are added to dE one by one with atomics (hot_bucket_kernel).
constexpr int64_t kMinPairBudget = int64_t(1) << 22;
constexpr int kMaxSlices = 32;
constexpr int kSliceHot = -1;                   // slice_of[] of a bucket that stays out of the index

// The pairs of a block's chunk, kPairBatch per thread at a time: all mask bytes are requested first, then ids and
// targets of the valid positions only (entries of padded positions are never read), so a thread waits for two round
// trips per batch instead of three per pair.  Sampled negatives are drawn again here instead of being read.  Fewer than 2^31 pairs on this path: 32-bit pair arithmetic.
constexpr int kPairBatch = 8;
static_assert(kChunkPairs % (kThreads * kPairBatch) == 0, "whole batches per chunk");

template <typename F>
__device__ __forceinline__ void for_live_pairs(const InvertArgs &a, int64_t chunk, F &&visit)
{
    const uint32_t p0 = (uint32_t)chunk * kChunkPairs, total = (uint32_t)(a.N * a.K), K = (uint32_t)a.K;
    for (int u0 = threadIdx.x; u0 < kChunkPairs; u0 += kThreads * kPairBatch) {
        uint32_t pos[kPairBatch];
        bool live[kPairBatch];
        int32_t id[kPairBatch], ti[kPairBatch];
#pragma unroll
        for (int j = 0; j < kPairBatch; ++j) {
            const uint32_t pair = p0 + u0 + j * kThreads;
            pos[j] = pair / K;
            live[j] = pair < total && (a.mask == nullptr || a.mask[pos[j]] != 0);
        }
#pragma unroll
        for (int j = 0; j < kPairBatch; ++j) {
            id[j] = ti[j] = 0;
            if (live[j]) {
                const uint32_t pair = p0 + u0 + j * kThreads;
                id[j] = a.smp.kind ? sample1(a.smp, pos[j], pair - pos[j] * K + 1u) : a.neg[pair];  // slot s is draw s + 1
                ti[j] = a.tgt[pos[j]];
            }
        }
#pragma unroll
        for (int j = 0; j < kPairBatch; ++j) {
            if (a.validate && (ti[j] < 0 || (int64_t)ti[j] >= a.V || id[j] < 0 || (int64_t)id[j] >= a.V)) live[j] = false;  // flagged elsewhere
            if (a.collide && id[j] == ti[j]) live[j] = false;
            if (live[j]) visit(id[j], (int32_t)pos[j]);
        }
    }
}

__global__ __launch_bounds__(kThreads) void part_count_kernel(InvertArgs a)
{
    __shared__ int32_t hist[kMaxBuckets];
    for (int b = threadIdx.x; b < a.n_buckets; b += kThreads) hist[b] = 0;
    __syncthreads();
    for (int64_t chunk = blockIdx.x; chunk < a.n_chunks; chunk += gridDim.x)
        for_live_pairs(a, chunk, [&](int32_t id, int32_t) { atomicAdd(&hist[id >> kBucketShift], 1); });
    __syncthreads();
    for (int b = threadIdx.x; b < a.n_buckets; b += kThreads) a.part_hist[(int64_t)b * gridDim.x + blockIdx.x] = hist[b];
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.part_total = 0;  // last entry of the scanned array: receives the grand total
}

// Cuts the buckets into slices (see above) from the scanned (bucket, block) counts: slice_of[b], the start of every
// bucket inside its slice's arrays, and the cleared work-list counters of the slices.  One block.
__global__ __launch_bounds__(kScanThreads) void plan_slices_kernel(InvertArgs a)
{
    __shared__ int32_t lds[kScanThreads / 64 + 1];
    __shared__ int32_t base[kMaxSlices], lo[kMaxSlices], hi[kMaxSlices], any_hot;
    constexpr int PER = kMaxBuckets / kScanThreads;
    const int64_t nb = a.n_part_blocks;
    int32_t cnt[PER], cum[PER], sum = 0;
    bool hot[PER];
    for (int j = threadIdx.x; j < kMaxSlices; j += kScanThreads) {
        base[j] = lo[j] = 0x7fffffff;
        hi[j] = -1;
        a.slice_hot[j] = 0;
    }
    if (threadIdx.x == 0) any_hot = 0;
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        const int b = threadIdx.x * PER + t;
        cnt[t] = 0;
        if (b < a.n_buckets) {
            const int32_t s0 = a.part_hist[(int64_t)b * nb];
            const int32_t s1 = (b + 1 < a.n_buckets) ? a.part_hist[(int64_t)(b + 1) * nb] : a.part_total[0];
            cnt[t] = s1 - s0;
        }
        hot[t] = a.n_slices > 1 && (int64_t)cnt[t] > a.budget / 8;
        cum[t] = sum;                  // running count of the ordinary buckets in front of this one, within the thread
        if (!hot[t]) sum += cnt[t];
    }
    int32_t total;
    const int32_t before = block_exclusive_scan(sum, lds, total);
    const int32_t per_slice = (total + a.n_slices - 1) / a.n_slices > 0 ? (total + a.n_slices - 1) / a.n_slices : 1;
    int32_t sl[PER];
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        cum[t] += before;
        sl[t] = hot[t] ? kSliceHot : min(cum[t] / per_slice, a.n_slices - 1);
        const int b = threadIdx.x * PER + t;
        if (b < a.n_buckets && !hot[t]) {
            atomicMin(&base[sl[t]], cum[t]);
            atomicMin(&lo[sl[t]], b);
            atomicMax(&hi[sl[t]], b);
        }
        if (b < a.n_buckets && hot[t]) any_hot = 1;
    }
    __syncthreads();
    // buckets [slice_lo, slice_hi] of a slice (an empty slice has hi < lo), and whether any bucket stays out of the index
    for (int j = threadIdx.x; j < kMaxSlices; j += kScanThreads) {
        a.slice_hot[kMaxSlices + j] = lo[j];
        a.slice_hot[2 * kMaxSlices + j] = hi[j];
    }
    if (threadIdx.x == 0) a.slice_hot[3 * kMaxSlices] = any_hot;
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        const int b = threadIdx.x * PER + t;
        if (b < a.n_buckets) {
            a.slice_of[b] = sl[t];
            a.bucket_start[b] = hot[t] ? 0 : cum[t] - base[sl[t]];
        }
    }
}

// D_SC != 0: the first sc_blocks blocks scatter the gradient rows of the correct items (hidden size D_SC) instead;
// nothing in this launch or the next reads or writes dE, and their latency hides under the filing of the pairs.
template <int D_SC>
__global__ __launch_bounds__(kThreads) void part_scatter_kernel(InvertArgs a, TileArgs sc, int64_t sc_blocks)
{
    __shared__ int32_t cur[kMaxBuckets];
    static_assert(kThreads == kPosChunk && kMaxBuckets * 4 >= kPosChunk * 8, "the scatter role sorts 256 keys in this array");
    if (D_SC != 0 && (int64_t)blockIdx.x < sc_blocks) {
        pos_scatter_block<(D_SC != 0 ? D_SC : 64)>(sc, (int64_t)blockIdx.x, reinterpret_cast<uint64_t *>(cur));
        return;
    }
    // Buckets of this slice: the block's cursor starts at the block's scanned offset inside the bucket, moved to where
    // the bucket starts in the slice's arrays.  Buckets of other slices get a negative cursor and are skipped.
    const int64_t blk = (int64_t)blockIdx.x - (D_SC != 0 ? sc_blocks : 0);
    const int64_t nb = a.n_part_blocks;
    for (int b = threadIdx.x; b < a.n_buckets; b += kThreads)
        cur[b] = (a.slice_of[b] == a.slice) ? a.part_hist[(int64_t)b * nb + blk] - a.part_hist[(int64_t)b * nb] + a.bucket_start[b] : -1;
    __syncthreads();
    for (int64_t chunk = blk; chunk < a.n_chunks; chunk += nb)
        for_live_pairs(a, chunk, [&](int32_t id, int32_t pos) {
            int32_t *c = &cur[id >> kBucketShift];
            if (*c >= 0) a.tmp[atomicAdd(c, 1)] = make_int2(id, pos);  // cursors only grow: the sign never changes
        });
}

// Pairs of the buckets that stay out of the index (more than an eighth of the budget in 2048 consecutive ids): each is
// scored and added to dE on its own, one thread per pair, d atomics.  A correctness path for extreme skew, not a fast one.
template <typename T>
__global__ __launch_bounds__(kThreads) void hot_bucket_kernel(InvertArgs a)
{
    __shared__ int8_t is_hot[kMaxBuckets];
    if (a.slice_hot[3 * kMaxSlices] == 0) return;  // no such bucket (block-uniform)
    for (int b = threadIdx.x; b < a.n_buckets; b += kThreads) is_hot[b] = a.slice_of[b] == kSliceHot;
    __syncthreads();
    const T *Hp = static_cast<const T *>(a.H), *Ep = static_cast<const T *>(a.E);
    for (int64_t chunk = blockIdx.x; chunk < a.n_chunks; chunk += gridDim.x)
        for_live_pairs(a, chunk, [&](int32_t id, int32_t pos) {
            if (!is_hot[id >> kBucketShift]) return;
            const T *h = Hp + (int64_t)pos * a.d, *e = Ep + (int64_t)id * a.d;
            float o = 0.f;
            for (int t = 0; t < a.d; ++t) o = fmaf(load1(h + t), load1(e + t), o);
            const float G = (a.g ? a.g[pos] : 1.f) * fast_exp(o - a.lse_in[pos]);
            float *row = a.dE + (int64_t)id * a.d;
            for (int t = 0; t < a.d; ++t) unsafeAtomicAdd(row + t, G * load1(h + t));
        });
}

__global__ __launch_bounds__(kScanThreads) void bucket_sort_kernel(InvertArgs a)
{
    __shared__ int32_t hist[kBucketIds];
    __shared__ int32_t lds[kScanThreads / 64 + 1];
    const int b = blockIdx.x;
    if (a.slice_of[b] != a.slice) return;  // block-uniform
    const int64_t n_blocks1 = a.n_part_blocks;
    // the bucket's range in tmp: it starts where the slice plan put it and holds as many pairs as the scanned (bucket,
    // block 0) entries of this bucket and the next are apart
    const int32_t s0 = a.part_hist[(int64_t)b * n_blocks1];
    const int32_t s1 = (b + 1 < a.n_buckets) ? a.part_hist[(int64_t)(b + 1) * n_blocks1] : a.part_total[0];
    const int32_t rb = a.bucket_start[b];
    const int32_t re = rb + (s1 - s0);
    const int64_t id0 = (int64_t)b << kBucketShift;
    for (int k = threadIdx.x; k < kBucketIds; k += kScanThreads) hist[k] = 0;
    __syncthreads();
    // A hot item owns most entries of its bucket, and 64 lanes adding to one LDS word take 64 turns: in a crowded bucket
    // the lanes that hold the same id as the first active lane are counted with one ballot and added by that lane alone.
    const bool crowded = re - rb > 16 * kBucketIds;  // block-uniform; ordinary buckets take the plain loops
    if (!crowded)
        for (int32_t e = rb + (int32_t)threadIdx.x; e < re; e += kScanThreads) atomicAdd(&hist[a.tmp[e].x - (int32_t)id0], 1);
    for (int32_t e0 = rb; crowded && e0 < re; e0 += kScanThreads) {
        const int32_t e = e0 + (int32_t)threadIdx.x;
        const bool in = e < re;
        const int32_t k = in ? a.tmp[e].x - (int32_t)id0 : -1;
        const int32_t lead = __builtin_amdgcn_readfirstlane(k);
        const uint64_t same = __ballot(in && k == lead);
        if (in) {
            if (k == lead) {
                if ((same & ((1ull << (threadIdx.x & 63)) - 1ull)) == 0) atomicAdd(&hist[k], (int32_t)__popcll(same));
            } else {
                atomicAdd(&hist[k], 1);
            }
        }
    }
    __syncthreads();
    // exclusive scan over the counts: consecutive ids per thread
    int32_t v[kBucketIds / kScanThreads], sum = 0;
#pragma unroll
    for (int t = 0; t < kBucketIds / kScanThreads; ++t) {
        v[t] = hist[threadIdx.x * (kBucketIds / kScanThreads) + t];
        sum += v[t];
    }
    int32_t total;
    int32_t run = block_exclusive_scan(sum, lds, total);
#pragma unroll
    for (int t = 0; t < kBucketIds / kScanThreads; ++t) {
        const int k = threadIdx.x * (kBucketIds / kScanThreads) + t;
        hist[k] = run;  // start of the item's segment inside the bucket; advanced below while filing
        run += v[t];
        if (id0 + k < a.V) a.cursor[id0 + k] = rb + run;  // END of the item's segment
    }
    __syncthreads();
    if (!crowded)
        for (int32_t e = rb + (int32_t)threadIdx.x; e < re; e += kScanThreads) {
            const int2 t = a.tmp[e];
            const int32_t slot = atomicAdd(&hist[t.x - (int32_t)id0], 1);
            a.pairs[rb + slot] = t.y;
        }
    for (int32_t e0 = rb; crowded && e0 < re; e0 += kScanThreads) {
        const int32_t e = e0 + (int32_t)threadIdx.x;
        const bool in = e < re;
        const int2 t = in ? a.tmp[e] : make_int2(-1, 0);
        const int32_t k = in ? t.x - (int32_t)id0 : -1;
        const int32_t lead = __builtin_amdgcn_readfirstlane(k);
        const uint64_t same = __ballot(in && k == lead);
        const int lane = threadIdx.x & 63;
        int32_t slot = 0;
        if (in && k == lead) {  // one returning add for all of them, ranks by lane order
            const int first = __ffsll((unsigned long long)same) - 1;
            int32_t base = 0;
            if (lane == first) base = atomicAdd(&hist[k], (int32_t)__popcll(same));
            base = __shfl(base, first, 64);
            slot = base + (int32_t)__popcll(same & ((1ull << lane) - 1ull));
        } else if (in) {
            slot = atomicAdd(&hist[k], 1);
        }
        if (in) a.pairs[rb + slot] = t.y;
    }
}

// Walks the positions filed in pairs[r, r_end) for the item whose row e the lane group holds, kInFlight at a time:
// recomputes each score against the hidden state (L2-resident), forms g exp(o - lse) and adds G h to acc.
// Every lane of the wavefront calls it (the loop condition is a wavefront vote, the scalar products use shuffles).
template <typename T, int LPR>
__device__ __forceinline__ void walk_segment(const InvertArgs &a, const float (&e)[8], int32_t r, int32_t r_end, bool col_ok,
                                             int c, float (&acc)[8])
{
    constexpr int U = RawChunk<T>::kInFlight;
    const T *Hp = static_cast<const T *>(a.H);
    while (__any(r < r_end)) {
        int32_t pos[U];
        RawChunk<T> raw[U];
        float lse[U], g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) pos[u] = (r + u < r_end) ? stream_load(a.pairs + r + u) : -1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            raw[u].clear();
            lse[u] = 0.f;
            g[u] = 0.f;
            if (pos[u] >= 0) {
                if (col_ok) raw[u].load(Hp + pos[u] * (int64_t)a.d + c * 8);
                lse[u] = a.lse_in[pos[u]];
                g[u] = a.g ? a.g[pos[u]] : 1.f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float h[8];
            raw[u].widen(h);
            float part = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) part = fmaf(h[t], e[t], part);
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) part += __shfl_xor(part, off, 64);  // partners share the item
            const float G = (pos[u] >= 0) ? g[u] * fast_exp(part - lse[u]) : 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[t] = fmaf(G, h[t], acc[t]);
        }
        r += U;
    }
}

// An item sampled by more than kHotPairs positions (popularity-weighted negatives: the head of the law collects
// percents of all pairs) would keep one lane group walking for milliseconds.  Its segment is cut into chunks of
// kHotPairs instead, filed in a work list, and hot_item_kernel spreads the chunks over the chip and adds their partial
// rows with atomics (d atomics per kHotPairs pairs).
constexpr int kHotPairs = 256;
constexpr int kItemBlocks = 16384;  // grid of the item pass over a slice

// One group of LPR lanes per item: e_v stays in registers, the positions that sampled it are walked four at a time.
template <typename T, int LPR>
__global__ __launch_bounds__(kThreads) void item_dE_kernel(InvertArgs a)
{
    constexpr int GPW = 64 / LPR;  // items per wavefront
    constexpr int IPB = (kThreads / 64) * GPW;  // items per block and trip
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const bool col_ok = c * 8 < a.d;
    // items of this launch: the whole table, or the buckets of the slice at hand (a fixed grid strides over them)
    int64_t v_lo = 0, v_hi = a.V;
    if (a.slice_of) {
        v_lo = (int64_t)a.slice_hot[kMaxSlices + a.slice] << kBucketShift;
        v_hi = min(a.V, ((int64_t)a.slice_hot[2 * kMaxSlices + a.slice] + 1) << kBucketShift);
    }
    for (int64_t v0 = v_lo + (int64_t)blockIdx.x * IPB; v0 < v_hi; v0 += (int64_t)gridDim.x * IPB) {
    const int64_t v = v0 + (threadIdx.x >> 6) * GPW + lane / LPR;
    int32_t r = 0, r_end = 0;
    if (v < v_hi && (a.slice_of == nullptr || a.slice_of[v >> kBucketShift] == a.slice)) {
        // cursor[v] is the end of item v's segment; it starts where the one before it ends, the first item of a bucket
        // where the bucket starts in the slice's arrays (without slices: one running array over all items)
        if (a.slice_of) r = ((v & (kBucketIds - 1)) == 0) ? a.bucket_start[v >> kBucketShift] : a.cursor[v - 1];
        else r = (v == 0) ? 0 : a.cursor[v - 1];
        r_end = a.cursor[v];
    }
    if (!__any(r < r_end)) continue;
    if (r_end - r > kHotPairs) {  // hot item: file its chunks and leave it to hot_item_kernel
        const int32_t n_chunks = (r_end - r + kHotPairs - 1) / kHotPairs;
        int32_t slot = 0;
        if (c == 0) slot = atomicAdd(a.hot_count, n_chunks);
        slot = __shfl(slot, lane - c, 64);
        for (int32_t k = c; k < n_chunks; k += LPR) {
            const int32_t b = r + k * kHotPairs;
            if (slot + k < a.hot_capacity) a.hot_list[slot + k] = make_int4((int32_t)v, b, min(b + kHotPairs, r_end), 0);
        }
        r = r_end = 0;
    }
    float e[8], acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) e[t] = acc[t] = 0.f;
    // the item row and the dE row it will be added to are requested together, before the walk over the positions
    const bool mine = r < r_end && col_ok;
    float4 *row = reinterpret_cast<float4 *>(a.dE + (mine ? v : 0) * (int64_t)a.d + c * 8);
    float4 dx = make_float4(0.f, 0.f, 0.f, 0.f), dy = dx;
    if (mine) {  // used once each: they must not push the hidden states out of L2
        stream_load8(static_cast<const T *>(a.E) + v * (int64_t)a.d + c * 8, e);
        dx = stream_load(row);
        dy = stream_load(row + 1);
    }
    walk_segment<T, LPR>(a, e, r, r_end, col_ok, c, acc);
    // the row belongs to this lane group alone: plain read-modify-write
    if (mine) {
        dx.x += acc[0]; dx.y += acc[1]; dx.z += acc[2]; dx.w += acc[3];
        dy.x += acc[4]; dy.y += acc[5]; dy.z += acc[6]; dy.w += acc[7];
        stream_store(row, dx);
        stream_store(row + 1, dy);
    }
    }  // item groups of this block
}

// The chunks item_dE_kernel filed: one lane group per chunk, a fixed grid strides over the list.
constexpr int kHotBlocks = 1024;
template <typename T, int LPR>
__global__ __launch_bounds__(kThreads) void hot_item_kernel(InvertArgs a)
{
    constexpr int GPW = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const bool col_ok = c * 8 < a.d;
    const int32_t n = min(*a.hot_count, a.hot_capacity);
    const int32_t stride = (int32_t)gridDim.x * (kThreads / 64) * GPW;
    for (int32_t e0 = ((int32_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) * GPW; e0 < n; e0 += stride) {
        const int32_t ent = e0 + lane / LPR;  // e0 is the same for the whole wavefront
        int32_t v = 0, r = 0, r_end = 0;
        if (ent < n) {
            const int4 t = a.hot_list[ent];
            v = t.x;
            r = t.y;
            r_end = t.z;
        }
        float e[8], acc[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) e[t] = acc[t] = 0.f;
        const bool mine = r < r_end && col_ok;
        if (mine) load8(static_cast<const T *>(a.E) + v * (int64_t)a.d + c * 8, e);
        walk_segment<T, LPR>(a, e, r, r_end, col_ok, c, acc);
        if (mine) {
            float *row = a.dE + v * (int64_t)a.d + c * 8;
#pragma unroll
            for (int t = 0; t < 8; ++t) unsafeAtomicAdd(row + t, acc[t]);
        }
    }
}

template <typename T, int LPR>
hipError_t launch_item_dE(const InvertArgs &a, hipStream_t stream)
{
    constexpr int items_per_block = (kThreads / 64) * (64 / LPR);
    ProfScope prof(PROF_ITEM_DE, stream);
    if (!a.slice_of) {  // the sliced index build has cleared the work-list counters on its way (plan_slices_kernel)
        const hipError_t e = launch_fill_zero(a.hot_count, 1, stream);
        if (e != hipSuccess) return e;
    }
    // unsliced: one trip per block; sliced: the slice's item range is only known on the device, a grid of at most
    // kItemBlocks strides over it
    int64_t item_blocks = (a.V + items_per_block - 1) / items_per_block;
    if (a.slice_of && item_blocks > kItemBlocks) item_blocks = kItemBlocks;
    hipLaunchKernelGGL((item_dE_kernel<T, LPR>), dim3((unsigned)item_blocks), dim3(kThreads), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((hot_item_kernel<T, LPR>), dim3(kHotBlocks), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_item_dE_by_width(const InvertArgs &a, hipStream_t stream)
{
    const int chunks = (a.d + 7) / 8;
    if (chunks <= 2) return launch_item_dE<T, 2>(a, stream);
    if (chunks <= 4) return launch_item_dE<T, 4>(a, stream);
    if (chunks <= 8) return launch_item_dE<T, 8>(a, stream);
    if (chunks <= 16) return launch_item_dE<T, 16>(a, stream);
    if (chunks <= 32) return launch_item_dE<T, 32>(a, stream);
    return launch_item_dE<T, 64>(a, stream);
}

// One thread per four consecutive draws of a position.
__global__ __launch_bounds__(kThreads) void sample_kernel(Sampler smp, int64_t n_pos, int32_t K, int32_t *out)
{
    const int64_t quads = ((int64_t)K + 4) / 4;  // draws 0..K cover K/4 + 1 groups of four
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_pos * quads) return;
    const int64_t i = t / quads;
    const uint32_t q4 = (uint32_t)(t - i * quads);
    int32_t id[4];
    sample4(smp, (uint64_t)i, q4, id);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int64_t j = 4 * (int64_t)q4 + w;  // draw number; slot j - 1
        if (j >= 1 && j <= K) out[i * K + (j - 1)] = id[w];
    }
}

}  // namespace

hipError_t launch_sample(const Sampler &smp, int64_t n_pos, int32_t K, int32_t *out, hipStream_t stream)
{
    const int64_t threads = n_pos * (((int64_t)K + 4) / 4);
    if (n_pos <= 0 || K <= 0) return hipSuccess;
    hipLaunchKernelGGL(sample_kernel, dim3((unsigned)((threads + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, smp, n_pos, K, out);
    return hipGetLastError();
}

int64_t invert_pair_budget(int64_t N, int64_t K)
{
    const int64_t pairs = N * K, eighth = (pairs + 7) / 8;
    return eighth > kMinPairBudget ? eighth : kMinPairBudget;
}
int invert_slices(int64_t N, int64_t K)
{
    const int64_t pairs = N * K, B = invert_pair_budget(N, K), room = B - B / 8;
    return pairs <= B ? 1 : (int)((pairs + room - 1) / room);
}
int64_t invert_index_pairs(int64_t N, int64_t K)   // entries of the arrays the index is filed into
{
    const int64_t pairs = N * K, B = invert_pair_budget(N, K);
    return pairs < B ? pairs : B;
}
size_t invert_hot_capacity(int64_t N, int64_t K) { return (size_t)(2 * (invert_index_pairs(N, K) / kHotPairs) + 16); }
size_t invert_scan_blocks(int64_t n) { return (size_t)((n + kScanChunk - 1) / kScanChunk); }
int64_t invert_part_blocks(int64_t N, int64_t K)
{
    const int64_t chunks = (N * K + kChunkPairs - 1) / kChunkPairs;
    return chunks < kMaxPartBlocks ? chunks : kMaxPartBlocks;
}
int64_t invert_buckets(int64_t V) { return (V + kBucketIds - 1) / kBucketIds; }
bool invert_partitioned(int64_t V) { return invert_buckets(V) <= kMaxBuckets; }
int invert_plan_words() { return 3 * kMaxSlices + 8; }  // work-list counters, first and last bucket of every slice, one flag

hipError_t launch_inverted_dE(bool bf16, const InvertArgs &a_in, const TileArgs *scatter, hipStream_t stream)
{
    InvertArgs a = a_in;
    if (a.N == 0) return hipSuccess;
    if (a.K == 0) return scatter ? launch_pos_scatter(*scatter, stream) : hipSuccess;
    const int64_t pairs = a.N * a.K;
    hipError_t e;
    auto check = [&]() { return (e = hipGetLastError()) == hipSuccess; };
    if (!invert_partitioned(a.V)) {
        // catalogue too large for the LDS bucket histogram (the caller only comes here when all pairs fit the budget):
        // counting sort with integer atomics on the V-word table, one running array over all items
        a.slice_of = nullptr;
        a.bucket_start = nullptr;
        {
            ProfScope prof(PROF_INDEX, stream);
            if (scatter && (e = launch_pos_scatter(*scatter, stream)) != hipSuccess) return e;
            const unsigned pair_blocks = (unsigned)((pairs + kThreads - 1) / kThreads);
            if ((e = launch_fill_zero(a.cursor, (size_t)a.V, stream)) != hipSuccess) return e;
            hipLaunchKernelGGL(count_kernel, dim3(pair_blocks), dim3(kThreads), 0, stream, a);
            if (!check()) return e;
            if ((e = launch_scan(a.cursor, a.V, a.block_sums, stream)) != hipSuccess) return e;
            hipLaunchKernelGGL(fill_kernel, dim3(pair_blocks), dim3(kThreads), 0, stream, a);
            if (!check()) return e;
        }
        return bf16 ? launch_item_dE_by_width<uint16_t>(a, stream) : launch_item_dE_by_width<float>(a, stream);
    }
    a.n_buckets = (int32_t)invert_buckets(a.V);
    a.n_part_blocks = invert_part_blocks(a.N, a.K);
    a.n_chunks = (pairs + kChunkPairs - 1) / kChunkPairs;
    a.budget = invert_pair_budget(a.N, a.K);
    a.n_slices = invert_slices(a.N, a.K);
    if (a.n_slices > kMaxSlices) return hipErrorInvalidValue;  // cannot happen: at most 11 by construction
    const int64_t n_hist = (int64_t)a.n_buckets * a.n_part_blocks;
    a.part_total = a.part_hist + n_hist;  // one extra word: scanning n_hist + 1 entries leaves the grand total there
    {
        ProfScope prof(PROF_INDEX, stream);
        hipLaunchKernelGGL(part_count_kernel, dim3((unsigned)a.n_part_blocks), dim3(kThreads), 0, stream, a);
        if (!check()) return e;
        if ((e = launch_scan(a.part_hist, n_hist + 1, a.block_sums, stream)) != hipSuccess) return e;
        hipLaunchKernelGGL(plan_slices_kernel, dim3(1), dim3(kScanThreads), 0, stream, a);
        if (!check()) return e;
    }
    for (int32_t j = 0; j < a.n_slices; ++j) {
        a.slice = j;
        a.hot_count = a.slice_hot + j;
        {
            ProfScope prof(PROF_INDEX, stream);
            if (scatter && j == 0) {  // the correct items' rows ride at the head of the first filing launch
                const int64_t sc_blocks = (scatter->N + kPosChunk - 1) / kPosChunk;
                const dim3 grid((unsigned)(a.n_part_blocks + sc_blocks));
                switch (scatter->d) {
                case 64: hipLaunchKernelGGL(part_scatter_kernel<64>, grid, dim3(kThreads), 0, stream, a, *scatter, sc_blocks); break;
                case 128: hipLaunchKernelGGL(part_scatter_kernel<128>, grid, dim3(kThreads), 0, stream, a, *scatter, sc_blocks); break;
                case 256: hipLaunchKernelGGL(part_scatter_kernel<256>, grid, dim3(kThreads), 0, stream, a, *scatter, sc_blocks); break;
                default: return hipErrorInvalidValue;
                }
            } else {
                hipLaunchKernelGGL(part_scatter_kernel<0>, dim3((unsigned)a.n_part_blocks), dim3(kThreads), 0, stream, a, TileArgs{}, 0);
            }
            if (!check()) return e;
            hipLaunchKernelGGL(bucket_sort_kernel, dim3((unsigned)a.n_buckets), dim3(kScanThreads), 0, stream, a);
            if (!check()) return e;
        }
        e = bf16 ? launch_item_dE_by_width<uint16_t>(a, stream) : launch_item_dE_by_width<float>(a, stream);
        if (e != hipSuccess) return e;
    }
    if (a.n_slices > 1) {  // buckets too crowded for any slice, if there are any
        ProfScope prof(PROF_ITEM_DE, stream);
        if (bf16) hipLaunchKernelGGL(hot_bucket_kernel<uint16_t>, dim3((unsigned)a.n_part_blocks), dim3(kThreads), 0, stream, a);
        else hipLaunchKernelGGL(hot_bucket_kernel<float>, dim3((unsigned)a.n_part_blocks), dim3(kThreads), 0, stream, a);
        if (!check()) return e;
    }
    return hipSuccess;
}

}  // namespace cce
