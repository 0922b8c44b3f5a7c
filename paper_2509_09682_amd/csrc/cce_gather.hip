// Row-gather kernels: one wavefront per position, candidate rows fetched one by one.
//
// This is the data access scheme of the paper's Alg. 1 / Alg. 2 as printed: for a block of positions, walk the
// candidate columns j of the index matrix, load the indexed item rows, take the scalar product over the whole hidden
// dimension (never split, Sec. 3.3), and keep the running max / sum of the online softmax on chip.  It serves every
// mode and dtype; it is the fast path for per-position negatives (a batched GEMV with no operand reuse, bound by the
// row gathers) and the exact-fp32 path.
//
// Lane layout: a row of d elements is covered by LPR lanes, 8 consecutive elements (one 16-byte bf16 load) per lane, so
// a wavefront scores 64/LPR candidates per load instruction and UNROLL of those are in flight together.  The dot
// product is finished with a butterfly over the LPR lanes.  dE updates use a second, interleaved column mapping
// (lane c owns columns c, c+LPR, ...) so that one atomic instruction covers consecutive addresses of the row.
#include <type_traits>

#include "cce_device.hpp"
#include "cce_kernels.hpp"

namespace cce {
namespace {

constexpr int kWavesPerBlock = 4;
// load instructions in flight per wavefront: bf16 rows stay packed in registers until they are used, so eight fit where
// four widened ones would
template <typename T> constexpr int unroll_of() { return RawChunk<T>::kInFlight; }
constexpr int kWindow = 256;  // per-position negatives: candidate ids a wavefront stages per refill of its LDS window

// Where the ids of the negatives come from.
enum { IDS_DIRECT = 0,   // shared list (or none): read where needed, every wavefront reads the same cached words
       IDS_STORED = 1,   // per-position list in memory: staged a window at a time with four coalesced loads
       IDS_SAMPLED = 2 };  // per-position draws of the counter-based sampler: generated a window at a time

// Per-position negatives: the wavefront fills its LDS window with the ids of candidates [j0, j0 + kWindow) of its
// position (candidate j >= 1 is slot j - 1 of the list, draw j of the sampler); candidate() reads them from there,
// so the row gathers never wait for a scattered 4-byte load first.  Sampled: four consecutive draws per lane from one
// or two generator calls.  LDS operations of one wavefront complete in order, so the reads that follow see the writes.
template <int IDS>
__device__ __forceinline__ void refill_window(const Params &p, int64_t i, int64_t j0, int32_t *win)
{
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_wave_barrier();
    if (IDS == IDS_SAMPLED) {
        int32_t id[4];
        sample4(p.smp, (uint64_t)i, (uint32_t)(j0 >> 2) + lane, id);
        *reinterpret_cast<int4 *>(win + 4 * lane) = make_int4(id[0], id[1], id[2], id[3]);
    } else {
        int32_t id[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t j = j0 + t * 64 + lane;
            id[t] = (j >= 1 && j <= p.K) ? p.neg[i * (int64_t)p.K + (j - 1)] : 0;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) win[t * 64 + lane] = id[t];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int LPR>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Candidate j of position i: id, whether it is the correct item, whether it takes part.
struct Cand {
    int64_t id;
    bool is_pos;
    bool live;
};

template <int IDS>
__device__ __forceinline__ Cand candidate(const Params &p, int64_t i, int64_t j, int64_t n_cand, int32_t ti, bool &bad,
                                          const int32_t *win)
{
    Cand c{0, false, false};
    if (j >= n_cand) return c;
    if (p.neg_mode == CCE_NEG_FULL) {
        c.id = j;
        c.is_pos = (j == ti);
        c.live = true;
        return c;
    }
    if (j == 0) {
        c.id = ti;
        c.is_pos = true;
        c.live = true;
        return c;
    }
    const int32_t id = (IDS != IDS_DIRECT) ? win[j & (kWindow - 1)]
                                           : ((p.neg_mode == CCE_NEG_SHARED) ? p.neg[j - 1] : p.neg[i * (int64_t)p.K + (j - 1)]);
    c.id = id;
    c.live = !(p.collide && id == ti);
    if (p.validate && (id < 0 || (int64_t)id >= p.V)) {
        c.live = false;
        bad = true;
    }
    return c;
}

template <typename T, int LPR, int IDS>
__global__ __launch_bounds__(kWavesPerBlock * 64) void fwd_gather_kernel(Params p)
{
    constexpr int RPI = 64 / LPR;  // candidate rows per wavefront step
    constexpr int kUnroll = unroll_of<T>();
    static_assert(kWindow % (RPI * kUnroll) == 0, "a step never straddles two windows");
    __shared__ int32_t window[IDS != IDS_DIRECT ? kWavesPerBlock : 1][IDS != IDS_DIRECT ? kWindow : 1];
    int32_t *win = window[IDS != IDS_DIRECT ? (threadIdx.x >> 6) : 0];
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int grp = lane / LPR;
    const int64_t i = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (i >= p.N) return;

    bool valid = (p.mask == nullptr) || (p.mask[i] != 0);
    int32_t ti = 0;
    bool bad = false;
    if (valid) {
        ti = p.tgt[i];
        if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) { bad = true; valid = false; }
    }
    if (!valid) {
        if (lane == 0) {
            p.loss[i] = 0.f;
            p.lse[i] = 0.f;
            if (bad) atomicOr(p.status, 1);
        }
        return;
    }

    const T *Hp = static_cast<const T *>(p.H);
    const T *Ep = static_cast<const T *>(p.E);
    const bool col_ok = (c * 8 < p.d);
    float h[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) h[t] = 0.f;
    if (col_ok) load8(Hp + i * (int64_t)p.d + c * 8, h);

    const int64_t n_cand = (p.neg_mode == CCE_NEG_FULL) ? p.V : (int64_t)p.K + 1;
    float m = -INFINITY, s = 0.f, o_pos = 0.f;

    for (int64_t j0 = 0; j0 < n_cand; j0 += RPI * kUnroll) {
        if (IDS != IDS_DIRECT && (j0 & (kWindow - 1)) == 0) refill_window<IDS>(p, i, j0, win);
        Cand cd[kUnroll];
        RawChunk<T> raw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            cd[u] = candidate<IDS>(p, i, j0 + u * RPI + grp, n_cand, ti, bad, win);
            raw[u].clear();
            if (cd[u].live && col_ok) raw[u].load(Ep + cd[u].id * (int64_t)p.d + c * 8);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float e[8];
            raw[u].widen(e);
            float part = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) part = fmaf(h[t], e[t], part);
            const float o = group_sum<LPR>(part);
            if (cd[u].live) {
                if (cd[u].is_pos) o_pos = o;
                const float mn = fmaxf(m, o);
                s = s * fast_exp(m - mn) + fast_exp(o - mn);  // first live step: exp(-inf) = 0
                m = mn;
            }
        }
    }
    // combine the 64/LPR candidate groups
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off, 64);
        const float s2 = __shfl_xor(s, off, 64);
        lse_merge(m, s, m2, s2);
        o_pos += __shfl_xor(o_pos, off, 64);
    }
    if (p.validate && __any(bad)) {
        if (lane == 0) atomicOr(p.status, 1);
    }
    if (lane == 0) {
        const float l = m + fast_log(s);
        p.lse[i] = l;
        p.loss[i] = l - o_pos;
    }
}


// Forward pass that also forms the hidden-state gradient short of the upstream gradient (fuse_dH on this family): the
// candidate rows are in registers once, for the score; the same visit adds softmax-weighted rows up (an online softmax
// carried through Eq. 6 left), so the backward call gathers no candidate row for dH at all.  Each lane group takes the
// score of its first live candidate as the reference of its exponentials (any reference gives the same result as long
// as nothing leaves the float range) and never looks at a maximum again; the true maximum is tracked on the side, and
// if a sum did leave the range (a later score more than about 69 nats above the reference) the wavefront walks its
// candidates once more against that maximum.  Groups are merged at the end, each scaled from its own reference.
template <typename T, int LPR, int IDS>
__global__ __launch_bounds__(kWavesPerBlock * 64) void fwd_fused_gather_kernel(Params p)
{
    constexpr int RPI = 64 / LPR;
    constexpr int kUnroll = unroll_of<T>();
    static_assert(kWindow % (RPI * kUnroll) == 0, "a step never straddles two windows");
    __shared__ int32_t window[IDS != IDS_DIRECT ? kWavesPerBlock : 1][IDS != IDS_DIRECT ? kWindow : 1];
    int32_t *win = window[IDS != IDS_DIRECT ? (threadIdx.x >> 6) : 0];
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int grp = lane / LPR;
    const int64_t i = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (i >= p.N) return;

    bool valid = (p.mask == nullptr) || (p.mask[i] != 0);
    int32_t ti = 0;
    bool bad = false;
    if (valid) {
        ti = p.tgt[i];
        if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) { bad = true; valid = false; }
    }
    if (!valid) {  // the backward call writes the zero dH row of a padded position itself
        if (lane == 0) {
            p.loss[i] = 0.f;
            p.lse[i] = 0.f;
            if (bad) atomicOr(p.status, 1);
        }
        return;
    }

    const T *Hp = static_cast<const T *>(p.H);
    const T *Ep = static_cast<const T *>(p.E);
    const bool col_ok = (c * 8 < p.d);
    float h[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) h[t] = 0.f;
    if (col_ok) load8(Hp + i * (int64_t)p.d + c * 8, h);

    const int64_t n_cand = (p.neg_mode == CCE_NEG_FULL) ? p.V : (int64_t)p.K + 1;
    float ref = -INFINITY, s = 0.f, o_pos = 0.f, top = -INFINITY;  // top: largest live score this lane group has seen
    float acc[8];
    // one walk over the candidates; FIXED: the reference is given (second walk), else the first live score of the group
    auto walk = [&](auto fixed_tag) {
        constexpr bool FIXED = decltype(fixed_tag)::value;
        s = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = 0.f;
        for (int64_t j0 = 0; j0 < n_cand; j0 += RPI * kUnroll) {
            if (IDS != IDS_DIRECT && (j0 & (kWindow - 1)) == 0) refill_window<IDS>(p, i, j0, win);
            Cand cd[kUnroll];
            RawChunk<T> raw[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                cd[u] = candidate<IDS>(p, i, j0 + u * RPI + grp, n_cand, ti, bad, win);
                raw[u].clear();
                if (cd[u].live && col_ok) raw[u].load(Ep + cd[u].id * (int64_t)p.d + c * 8);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float e[8];
                raw[u].widen(e);
                float part = 0.f;
#pragma unroll
                for (int t = 0; t < 8; ++t) part = fmaf(h[t], e[t], part);
                const float o = group_sum<LPR>(part);
                if (cd[u].live) {
                    if (cd[u].is_pos) o_pos = o;
                    if (!FIXED) {
                        top = fmaxf(top, o);
                        if (ref == -INFINITY) ref = o;
                    }
                    const float w = fast_exp(o - ref);
                    s += w;
#pragma unroll
                    for (int t = 0; t < 8; ++t) acc[t] = fmaf(w, e[t], acc[t]);
                }
            }
        }
    };
    walk(std::false_type{});
    {   // did any sum of the wavefront leave the float range?  (the rows are sums of at most s * max|e|)
        const bool over = !(s < 1.0e30f);
        if (__any(over)) {
            float M = top;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
            ref = M;  // every group live or not: exp(o - M) <= 1
            walk(std::true_type{});
        }
    }
    // merge the lane groups: each holds (reference, sum, row) of its share of the candidates
    float M = ref;  // -inf for a group that saw no live candidate
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    const float scale = (ref == -INFINITY) ? 0.f : fast_exp(ref - M);
    s *= scale;
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] *= scale;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        s += __shfl_xor(s, off, 64);
        o_pos += __shfl_xor(o_pos, off, 64);
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] += __shfl_xor(acc[t], off, 64);
    }
    if (p.validate && __any(bad)) {
        if (lane == 0) atomicOr(p.status, 1);
    }
    const float l = M + fast_log(s);
    const float inv = 1.f / s;
    if (lane == 0) {
        p.lse[i] = l;
        p.loss[i] = l - o_pos;
        p.coef[i] = fast_exp(o_pos - l) - 1.f;  // coefficient of the correct item, short of the upstream gradient
    }
    if (grp == 0 && col_ok) {
        float et[8];
        load8(Ep + (int64_t)ti * p.d + c * 8, et);
        float4 *out = reinterpret_cast<float4 *>(p.U + i * (int64_t)p.d + c * 8);
        out[0] = make_float4(fmaf(acc[0], inv, -et[0]), fmaf(acc[1], inv, -et[1]), fmaf(acc[2], inv, -et[2]), fmaf(acc[3], inv, -et[3]));
        out[1] = make_float4(fmaf(acc[4], inv, -et[4]), fmaf(acc[5], inv, -et[5]), fmaf(acc[6], inv, -et[6]), fmaf(acc[7], inv, -et[7]));
    }
}

// Backward side of the fused forward pass: dH_i = grad_loss_i U_i (zero rows for padded positions), eight columns per
// thread; and, where no aggregated scatter exists for the hidden size, the correct items' rows
// dE[tgt_i] += grad_loss_i (p+_i - 1) H_i by atomics, one wavefront per position.
__global__ __launch_bounds__(256) void gather_scale_kernel(Params p)
{
    const int cpr = p.d / 8;  // d is a multiple of 8
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t i = idx / cpr;
    const int c = (int)(idx % cpr);
    if (i >= p.N) return;
    bool valid = (p.mask == nullptr) || (p.mask[i] != 0);
    if (valid && p.validate) {
        const int32_t ti = p.tgt[i];
        valid = ti >= 0 && (int64_t)ti < p.V;
    }
    float v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = 0.f;
    if (valid) {
        const float g = p.g ? p.g[i] : 1.f;
        load8(p.U + i * (int64_t)p.d + c * 8, v);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] *= g;
    }
    if (p.dH_bf16) {
        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(p.dH) + i * (int64_t)p.d + c * 8) =
            make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    } else {
        float4 *out = reinterpret_cast<float4 *>(static_cast<float *>(p.dH) + i * (int64_t)p.d + c * 8);
        out[0] = make_float4(v[0], v[1], v[2], v[3]);
        out[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void pos_rows_dE_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= p.N) return;
    if (p.mask && p.mask[i] == 0) return;
    const int32_t ti = p.tgt[i];
    if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) return;
    const float G = (p.g ? p.g[i] : 1.f) * p.coef[i];
    const T *hrow = static_cast<const T *>(p.H) + i * (int64_t)p.d;
    float *row = p.dE + (int64_t)ti * p.d;
    for (int col = lane; col < p.d; col += 64) unsafeAtomicAdd(row + col, G * load1(hrow + col));
}

// ATOMIC_DE = false: dE comes from other passes (inverted index, aggregated scatter); this pass yields dH and the
// correct-item coefficients only.
template <typename T, int LPR, bool ATOMIC_DE, int IDS>
__global__ __launch_bounds__(kWavesPerBlock * 64) void bwd_gather_kernel(Params p)
{
    constexpr int RPI = 64 / LPR;
    constexpr int kUnroll = unroll_of<T>();
    __shared__ int32_t window[IDS != IDS_DIRECT ? kWavesPerBlock : 1][IDS != IDS_DIRECT ? kWindow : 1];
    int32_t *win = window[IDS != IDS_DIRECT ? (threadIdx.x >> 6) : 0];
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int grp = lane / LPR;
    const int64_t i = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (i >= p.N) return;

    const bool col_ok = (c * 8 < p.d);
    bool valid = (p.mask == nullptr) || (p.mask[i] != 0);
    int32_t ti = 0;
    bool bad = false;
    if (valid) {
        ti = p.tgt[i];
        if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) { bad = true; valid = false; }
    }
    float acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = 0.f;

    if (valid) {
        const T *Hp = static_cast<const T *>(p.H);
        const T *Ep = static_cast<const T *>(p.E);
        float h[8], h2[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            h[t] = 0.f;
            const int col = c + LPR * t;
            h2[t] = (ATOMIC_DE && col < p.d) ? load1(Hp + i * (int64_t)p.d + col) : 0.f;
        }
        if (col_ok) load8(Hp + i * (int64_t)p.d + c * 8, h);
        const float lse = p.lse_in[i];
        const float gi = p.g ? p.g[i] : 1.f;
        const int64_t n_cand = (p.neg_mode == CCE_NEG_FULL) ? p.V : (int64_t)p.K + 1;

        for (int64_t j0 = 0; j0 < n_cand; j0 += RPI * kUnroll) {
            if (IDS != IDS_DIRECT && (j0 & (kWindow - 1)) == 0) refill_window<IDS>(p, i, j0, win);
            Cand cd[kUnroll];
            RawChunk<T> raw[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                cd[u] = candidate<IDS>(p, i, j0 + u * RPI + grp, n_cand, ti, bad, win);
                raw[u].clear();
                if (cd[u].live && col_ok) raw[u].load(Ep + cd[u].id * (int64_t)p.d + c * 8);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float e[8];
                raw[u].widen(e);
                float part = 0.f;
#pragma unroll
                for (int t = 0; t < 8; ++t) part = fmaf(h[t], e[t], part);
                const float o = group_sum<LPR>(part);
                if (cd[u].live) {
                    const float pj = fast_exp(o - lse);
                    const float G = gi * (pj - (cd[u].is_pos ? 1.f : 0.f));
#pragma unroll
                    for (int t = 0; t < 8; ++t) acc[t] = fmaf(G, e[t], acc[t]);
                    if (cd[u].is_pos && p.coef && c == 0) p.coef[i] = G;
                    if (ATOMIC_DE && (cd[u].is_pos ? !p.skip_pos_dE : !p.skip_neg_dE)) {
                        float *row = p.dE + cd[u].id * (int64_t)p.d;
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const int col = c + LPR * t;
                            if (col < p.d) unsafeAtomicAdd(row + col, G * h2[t]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[t] += __shfl_xor(acc[t], off, 64);
        }
    }
    if (p.validate && __any(bad)) {
        if (lane == 0) atomicOr(p.status, 1);
    }
    if (grp == 0 && col_ok) {
        if (p.dH_bf16) {
            uint4 w;
            w.x = pack_bf16x2(acc[0], acc[1]);
            w.y = pack_bf16x2(acc[2], acc[3]);
            w.z = pack_bf16x2(acc[4], acc[5]);
            w.w = pack_bf16x2(acc[6], acc[7]);
            *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(p.dH) + i * (int64_t)p.d + c * 8) = w;
        } else {
            float4 *out = reinterpret_cast<float4 *>(static_cast<float *>(p.dH) + i * (int64_t)p.d + c * 8);
            out[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            out[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
    }
}


// dE of the negatives that all positions share (a shared list, or the whole catalogue), candidate by candidate.
// Walking positions and adding a row per (position, candidate) pair, as the pass above does, sends every position's
// update to the same few rows: same-address atomics complete one at a time, and the backward pass was ten to sixty
// times the forward pass (12,800 positions, K = 1024, fp32, d = 64: 11.7 ms against 0.18 ms).  Here a wavefront owns
// kCandRows candidates and a slice of the positions: it keeps the candidates' rows in registers, streams the hidden
// states of its slice (one load serves all its candidates), recomputes score and coefficient g_i exp(o - lse_i), sums
// G h_i in registers and adds one row per candidate and slice at the end (Eq. 6 right, summed over positions first).
// The correct items stay with the position-major pass (they differ per position).  In full-catalogue mode the
// candidate that is the position's correct item is left to that pass as a whole (its coefficient there is g (p - 1)).
constexpr int kCandRows = 4;
template <typename T, int LPR>
__global__ __launch_bounds__(kWavesPerBlock * 64) void cand_dE_kernel(Params p, int64_t n_cand, int64_t pos_per_slice)
{
    constexpr int RPI = 64 / LPR;
    constexpr int kUnroll = unroll_of<T>() / 2;
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    const int grp = lane / LPR;
    const bool col_ok = (c * 8 < p.d);
    const int64_t j0 = ((int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * kCandRows;
    if (j0 >= n_cand) return;
    const bool full = (p.neg_mode == CCE_NEG_FULL);
    const T *Hp = static_cast<const T *>(p.H);
    const T *Ep = static_cast<const T *>(p.E);

    int64_t id[kCandRows];
    bool ok[kCandRows];
    float e[kCandRows][8], acc[kCandRows][8];
#pragma unroll
    for (int r = 0; r < kCandRows; ++r) {
        const int64_t j = j0 + r;
        ok[r] = j < n_cand;
        id[r] = ok[r] ? (full ? j : (int64_t)p.neg[j]) : 0;
        if (!full && p.validate && (id[r] < 0 || id[r] >= p.V)) ok[r] = false;  // flagged by the position-major pass
        if (!ok[r]) id[r] = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) e[r][t] = acc[r][t] = 0.f;
        if (ok[r] && col_ok) load8(Ep + id[r] * (int64_t)p.d + c * 8, e[r]);
    }
    const bool drop_own = full || p.collide;  // a candidate equal to the position's correct item takes no part here

    const int64_t i_begin = (int64_t)blockIdx.y * pos_per_slice;
    const int64_t i_end = (i_begin + pos_per_slice < p.N) ? i_begin + pos_per_slice : p.N;
    for (int64_t i0 = i_begin; i0 < i_end; i0 += RPI * kUnroll) {  // uniform trip count: the butterflies need every lane
        RawChunk<T> raw[kUnroll];
        float nlse[kUnroll], gi[kUnroll];
        int32_t ti[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = i0 + u * RPI + grp;
            bool valid = i < i_end && ((p.mask == nullptr) || (p.mask[i] != 0));
            raw[u].clear();
            nlse[u] = 0.f;
            gi[u] = 0.f;  // a position that takes no part has coefficient zero
            ti[u] = -1;
            if (valid) {
                ti[u] = p.tgt[i];
                if (p.validate && (ti[u] < 0 || (int64_t)ti[u] >= p.V)) valid = false;
            }
            if (valid) {
                if (col_ok) raw[u].load(Hp + i * (int64_t)p.d + c * 8);
                nlse[u] = -p.lse_in[i];
                gi[u] = p.g ? p.g[i] : 1.f;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float h[8];
            raw[u].widen(h);
#pragma unroll
            for (int r = 0; r < kCandRows; ++r) {
                float part = 0.f;
#pragma unroll
                for (int t = 0; t < 8; ++t) part = fmaf(h[t], e[r][t], part);
                const float o = group_sum<LPR>(part);
                float G = gi[u] * fast_exp(o + nlse[u]);
                if (gi[u] == 0.f || (drop_own && id[r] == (int64_t)ti[u])) G = 0.f;  // (also keeps 0 * inf out)
#pragma unroll
                for (int t = 0; t < 8; ++t) acc[r][t] = fmaf(G, h[t], acc[r][t]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kCandRows; ++r) {
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[r][t] += __shfl_xor(acc[r][t], off, 64);
        }
        if (ok[r] && grp == 0 && col_ok) {
            float *row = p.dE + id[r] * (int64_t)p.d + c * 8;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (c * 8 + t < p.d) unsafeAtomicAdd(row + t, acc[r][t]);
        }
    }
}

template <typename T, int LPR>
hipError_t launch_cand(const Params &p, hipStream_t stream)
{
    const int64_t n_cand = (p.neg_mode == CCE_NEG_FULL) ? p.V : (int64_t)p.K;
    if (p.N == 0 || n_cand == 0) return hipSuccess;
    constexpr int RPI = 64 / LPR;
    const int64_t gx = (n_cand + kWavesPerBlock * kCandRows - 1) / (kWavesPerBlock * kCandRows);
    // about eight blocks per compute unit; a slice no shorter than a few trips of the position loop
    int64_t slices = (2048 + gx - 1) / gx;
    const int64_t min_slice = (int64_t)RPI * unroll_of<T>() * 2;
    if (slices > (p.N + min_slice - 1) / min_slice) slices = (p.N + min_slice - 1) / min_slice;
    if (slices < 1) slices = 1;
    if (slices > 65535) slices = 65535;
    const int64_t per = (p.N + slices - 1) / slices;
    slices = (p.N + per - 1) / per;
    ProfScope prof(PROF_GATHER_BWD, stream);
    hipLaunchKernelGGL((cand_dE_kernel<T, LPR>), dim3((unsigned)gx, (unsigned)slices), dim3(kWavesPerBlock * 64), 0, stream, p, n_cand, per);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_cand_by_width(const Params &p, hipStream_t stream)
{
    const int chunks = (p.d + 7) / 8;
    if (chunks <= 2) return launch_cand<T, 2>(p, stream);
    if (chunks <= 4) return launch_cand<T, 4>(p, stream);
    if (chunks <= 8) return launch_cand<T, 8>(p, stream);
    if (chunks <= 16) return launch_cand<T, 16>(p, stream);
    if (chunks <= 32) return launch_cand<T, 32>(p, stream);
    return launch_cand<T, 64>(p, stream);
}

template <typename T, int LPR>
hipError_t launch_pair(bool backward, const Params &p, hipStream_t stream)
{
    if (p.N == 0) return hipSuccess;
    const dim3 block(kWavesPerBlock * 64);
    const dim3 grid((unsigned)((p.N + kWavesPerBlock - 1) / kWavesPerBlock));
    ProfScope prof(backward ? PROF_GATHER_BWD : PROF_GATHER_FWD, stream);
    const int ids = p.smp.kind ? IDS_SAMPLED : ((p.neg_mode == CCE_NEG_PER_POSITION && p.K > 0) ? IDS_STORED : IDS_DIRECT);
    auto launch = [&](auto tag) {
        constexpr int IDS = decltype(tag)::value;
        if (backward && p.skip_neg_dE && p.skip_pos_dE)
            hipLaunchKernelGGL((bwd_gather_kernel<T, LPR, false, IDS>), grid, block, 0, stream, p);
        else if (backward)
            hipLaunchKernelGGL((bwd_gather_kernel<T, LPR, true, IDS>), grid, block, 0, stream, p);
        else if (p.U)
            hipLaunchKernelGGL((fwd_fused_gather_kernel<T, LPR, IDS>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((fwd_gather_kernel<T, LPR, IDS>), grid, block, 0, stream, p);
    };
    if (ids == IDS_SAMPLED) launch(std::integral_constant<int, IDS_SAMPLED>{});
    else if (ids == IDS_STORED) launch(std::integral_constant<int, IDS_STORED>{});
    else launch(std::integral_constant<int, IDS_DIRECT>{});
    return hipGetLastError();
}

template <typename T>
hipError_t launch_by_width(bool backward, const Params &p, hipStream_t stream)
{
    const int chunks = (p.d + 7) / 8;
    if (chunks <= 2) return launch_pair<T, 2>(backward, p, stream);
    if (chunks <= 4) return launch_pair<T, 4>(backward, p, stream);
    if (chunks <= 8) return launch_pair<T, 8>(backward, p, stream);
    if (chunks <= 16) return launch_pair<T, 16>(backward, p, stream);
    if (chunks <= 32) return launch_pair<T, 32>(backward, p, stream);
    return launch_pair<T, 64>(backward, p, stream);
}

}  // namespace

hipError_t launch_gather(bool backward, bool bf16, const Params &p, hipStream_t stream)
{
    return bf16 ? launch_by_width<uint16_t>(backward, p, stream) : launch_by_width<float>(backward, p, stream);
}

hipError_t launch_gather_scale(bool bf16, bool pos_rows, const Params &p, hipStream_t stream)
{
    if (p.N == 0) return hipSuccess;
    ProfScope prof(PROF_DH_SCALE, stream);
    const int64_t n = p.N * (int64_t)(p.d / 8);
    hipLaunchKernelGGL(gather_scale_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !pos_rows) return e;
    const dim3 grid((unsigned)((p.N + 3) / 4));
    if (bf16) hipLaunchKernelGGL(pos_rows_dE_kernel<uint16_t>, grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(pos_rows_dE_kernel<float>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_shared_dE(bool bf16, const Params &p, hipStream_t stream)
{
    if (p.neg_mode == CCE_NEG_PER_POSITION) return hipErrorInvalidValue;
    return bf16 ? launch_cand_by_width<uint16_t>(p, stream) : launch_cand_by_width<float>(p, stream);
}

}  // namespace cce
