// Matrix-core kernels for the dense cases: shared negatives and the full catalogue, bf16 inputs.
//
// With one list of negatives for the whole batch the indexed scalar products of Alg. 1 / Alg. 2 become the dense
// contraction H x E_neg^T; in full-catalogue mode (Sec. 3.1, Eq. 2) E_neg is the whole table.  One kernel template
// serves the three passes.  A "stationary" operand X lives in registers, one row per lane column, and a "streamed"
// operand Y goes through LDS in tiles shared by the four wavefronts of a workgroup:
//
//   FWD : X = hidden states,  Y = candidate rows.  S^T = Y X^T on the matrix cores, online max / sum-exp per lane (Alg. 1).
//   DH  : X = hidden states,  Y = candidate rows.  P^T = exp(S^T - LSE), dH^T += Y^T P^T          (Alg. 2, Eq. 6 left).
//   DE  : X = candidate rows, Y = hidden states.   G   = g exp(S - LSE),  dE_neg^T += Y^T G       (Alg. 2, Eq. 6 right).
//
// Scores are produced transposed (streamed index in the accumulator registers, stationary index on the lanes) so that
// the softmax reduction of FWD needs no cross-lane traffic until the very end, and so that the probability tile can be
// fed back as the B operand of the second product straight from registers: the permutation the accumulator layout
// imposes on the reduction index is matched by reading the A operand with the LDS transpose loads of gfx950.
//
// The correct item is not a column of the dense tile.  Its score is taken separately (the paper's correct-logit
// kernel) and enters with a per-position weight w_i = 1 - c_i, c_i = number of negatives equal to the position's own
// target: the dense tile counts those c_i copies, the definition wants the target exactly once, so
//   sum_live exp(o) = sum_k exp(o_ik) + w_i exp(o+_i),   coefficient of the correct item = g_i (w_i p+_i - 1).
// With collision masking off w_i = 1; in full-catalogue mode the target is already one of the columns and w_i = 0.
//
// This header holds the kernel template, its merges and the launch planning.  Every hidden size is instantiated in a
// file of its own (cce_tile_d64.hip, cce_tile_d128.hip, cce_tile_d256.hip), which keeps the build parallel; everything
// here sits in an unnamed namespace, so each of those files gets its own copy.
#pragma once
#include <atomic>

#include "cce_device.hpp"
#include "cce_kernels.hpp"
#include "cce_scatter.hpp"
#include "cce_tile_shared.hpp"

namespace cce {

template <int D>
hipError_t launch_pos_scatter_scale_d(const TileArgs &a, hipStream_t stream);  // defined at the end of this header

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));


// MODE_FDH: the forward pass and the hidden-state gradient in one pass over the candidates (see the FDH notes in tile_body).
enum { MODE_FWD = 0, MODE_DH = 1, MODE_DE = 2, MODE_FDH = 3 };

// Compile-time tags: a full streamed tile, or the short last tile whose missing rows are masked.
struct Full { static constexpr bool value = false; };
struct Ragged { static constexpr bool value = true; };
// Forward softmax of a tile: with the running maximum kept up to date (Exact), or against the maximum as it stood when
// the tile began (Lazy: no maximum, no rescaling; the caller repeats the tile exactly if a sum overflowed).
struct Exact { static constexpr bool lazy = false; };
struct Lazy { static constexpr bool lazy = true; };
// The two forms of an attempt at a block's streamed range in the fused forward + dH pass (see the FDH notes in tile_body).
struct FastTag { static constexpr bool exact = false; };
struct ExactTag { static constexpr bool exact = true; };

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);  // round to nearest even
    uint32_t u;
    __builtin_memcpy(&u, &b, 4);
    return u;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    bf16x8 r;
    __builtin_memcpy(&r, &v, 16);
    return r;
}

// Item row of candidate column k (identity in full-catalogue mode).
__device__ __forceinline__ int64_t item_row(const TileArgs &a, int64_t k)
{
    if (!a.neg) return k;
    int64_t id = a.neg[k];
    if (a.validate && (id < 0 || id >= a.V)) id = 0;  // flagged by the preparation kernel; never dereferenced
    return id;
}

// Dot product of the lane's half of a stationary row (chunks kk*16 + hi*8 .. +8) with the same chunks of another row.
template <int D>
__device__ __forceinline__ float half_row_dot(const uint4 (&xr)[D / 16], const uint16_t *other, int hi)
{
    float s = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
        const uint4 o = *reinterpret_cast<const uint4 *>(other + kk * 16 + hi * 8);
        s = fmaf(bf16_lo(xr[kk].x), bf16_lo(o.x), s);
        s = fmaf(bf16_hi(xr[kk].x), bf16_hi(o.x), s);
        s = fmaf(bf16_lo(xr[kk].y), bf16_lo(o.y), s);
        s = fmaf(bf16_hi(xr[kk].y), bf16_hi(o.y), s);
        s = fmaf(bf16_lo(xr[kk].z), bf16_lo(o.z), s);
        s = fmaf(bf16_hi(xr[kk].z), bf16_hi(o.z), s);
        s = fmaf(bf16_lo(xr[kk].w), bf16_lo(o.w), s);
        s = fmaf(bf16_hi(xr[kk].w), bf16_hi(o.w), s);
    }
    return s;
}

// XOR pattern of the 16-byte chunk position inside an unpadded LDS row of CPR chunks.  LDS serves 256 bytes per clock:
// a 128-bit read is done 16 lanes at a time, a 64-bit transpose read 32 lanes at a time, and either runs at full rate
// only if those lanes touch 256 distinct bytes modulo 256.
//   128-bit operand reads: 16 consecutive rows, one chunk each -> (row * CPR + chunk) mod 16 must take 16 values;
//   transpose reads: 4 consecutive rows x 4 consecutive chunks -> the 16 (row, chunk) slots must differ modulo 16.
// Rows of 8 chunks alternate between the two halves of a 256-byte line, so 3 swizzle bits do; longer rows all start
// on the same bank and need 4.  (Measured: 209-214 bytes per clock for both read kinds, against 125 with a pattern
// that is only distinct over 8 rows.)
template <int CPR>
__device__ __forceinline__ int swz(int row)
{
    return CPR == 8 ? ((((row >> 1) & 1) << 2) | ((row >> 2) & 3)) : (((row & 3) << 2) | ((row >> 2) & 3));
}

typedef const void __attribute__((address_space(1))) *global_cptr;
typedef void __attribute__((address_space(3))) *lds_ptr;
typedef s16x4 __attribute__((address_space(3))) *lds_v4;

// Largest of three floats in one instruction; the operands are never NaN here, so no canonicalisation is wanted.
__device__ __forceinline__ float max3(float x, float y, float z)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z));
    return r;
}

// Waits until at most K of the wavefront's vector-memory operations are outstanding (they complete in issue order).
template <int K>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(K) : "memory");
}

// Workgroup barrier without the memory fence of __syncthreads(), which would wait for every load in flight: the
// wavefront's own LDS reads are drained, loads into other buffers keep flying.  Visibility of landed direct-to-LDS
// data is the caller's business (wait_all_but before the barrier).
__device__ __forceinline__ void barrier_keep_loads()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Waits until all but the youngest `groups` load groups of the wavefront have landed.  A group is BASE + extras
// direct-to-LDS instructions, extras in {0, 1, 2}; groups beyond 2 are treated as 2 (waiting for more is always safe).
template <int BASE>
__device__ __forceinline__ void wait_all_but(int groups, int extras)
{
    if (groups <= 0) {
        wait_vm<0>();
    } else if (groups == 1) {
        if (extras == 0) wait_vm<BASE>();
        else if (extras == 1) wait_vm<BASE + 1>();
        else wait_vm<BASE + 2>();
    } else {
        if (extras == 0) wait_vm<2 * BASE>();
        else if (extras == 1) wait_vm<2 * BASE + 2>();
        else wait_vm<2 * BASE + 4>();
    }
}

// The same, ordered behind the instruction that produced `after` (an input the instruction does not read).
__device__ __forceinline__ float max3_after(float after, float x, float y, float z)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z), "v"(after));
    return r;
}

constexpr int kScaleChunks = 4;  // 32-byte pieces of dH per thread of a scaling block

// dH = grad_loss * U for the valid positions, zero rows for the padded ones: one lane per 8 columns, positions in their
// original order.  FILE_G: the first blocks also file the upstream gradient under the compacted index (second half of
// de_const), where a dE pass that does not stream it by row number finds it.
template <int D>
__device__ __forceinline__ void dh_scale_chunk(const TileArgs &a, int64_t chunk)
{
    constexpr int LPR = D / 8;
    const int64_t i = chunk / LPR;
    const int c = (int)(chunk % LPR);
    if (i >= a.N) return;
    bool valid = (a.pos_mask == nullptr) || (a.pos_mask[i] != 0);
    if (valid && a.validate) {  // a position with a target out of range counts as padding
        const int32_t ti = a.tgt[i];
        valid = ti >= 0 && (int64_t)ti < a.V;
    }
    float v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = 0.f;
    if (valid) {
        const float g = a.g ? a.g[i] : 1.f;
        load8(a.U + i * D + c * 8, v);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] *= g;
    }
    if (a.dH_bf16) {
        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.dH) + i * D + c * 8) =
            make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
    } else {
        float4 *out = reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + i * D + c * 8);
        out[0] = make_float4(v[0], v[1], v[2], v[3]);
        out[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// D: hidden size.  BY: streamed rows per LDS tile.  NW: wavefronts per block.  XG: groups of 32 stationary rows per
// wavefront (XG = 2 reads every streamed operand from LDS once for two matrix instructions).  MINB: blocks per
// compute unit the register budget is sized for.  NBUF: LDS tile buffers in the ring (2..4: separate arrays, main loop
// unrolled NBUF times, NBUF - 1 tiles in flight; 0: two buffers in one array and a single copy of the loop body).
// FILTER: gradient filtering of the backward passes (32 x 32 blocks of the softmax matrix below a threshold are skipped).
// DS: wavefronts that share a group of stationary rows in the backward passes; each of them forms the full score tile
// and keeps 1/DS of the output columns, which divides the accumulator registers by DS at the price of DS score products.
// LDS needs of one tile-kernel configuration (the kernel wrappers declare the arrays, the body gets pointers).
template <int D, int MODE, int BY, int NW, int XG, int NBUF, int DS>
struct TileGeom {
    static constexpr int TILE = BY * D;
    static constexpr int IDS = (BY < 64) ? 64 : BY;
    static constexpr int CONSTS = (MODE == MODE_DE) ? 2 * BY : 0;
    static constexpr int BUF = ((TILE + 2 * CONSTS + 2 * IDS + 511) / 512) * 512;  // 16-bit elements per buffer
    static constexpr int XPB = (NW / DS) * XG * 32;
    static constexpr int EPI_BYTES = NW * 32 * 33 * 4 + XPB * 8;
    static constexpr bool EPI_IN_TILES = (MODE == MODE_DE) && (NW == 4) && (TILE * 2 >= 2 * 32 * 33 * 4 + XPB * 8);
    static constexpr int BUF0 = (NBUF == 0) ? 2 * BUF : BUF;
    static constexpr int BUF1 = (NBUF >= 2) ? BUF : 8;
    static constexpr int BUF2 = (NBUF >= 3) ? BUF : 8;
    static constexpr int BUF3 = (NBUF >= 4) ? BUF : 8;
    static constexpr int EPI_OWN = (MODE == MODE_DE && !EPI_IN_TILES) ? EPI_BYTES / 4 : 4;  // floats
};

// ---------------------------------------------------------------------------------------------------------------------
// Last-round split of the dH pass.  With one block per compute unit and equal blocks, n_xb position blocks take
// ceil(n_xb / slots) rounds, and a last round of a few blocks costs as much as a full one (c5: 600 blocks on 256
// slots, 3 rounds for 2.34 rounds of work).  The blocks of a last round that fills at most half the chip split the
// candidate range S ways instead (S = slots / tail, at most kTailMaxSplits), write partial rows, and a small merge
// adds them up.  The count of valid positions is only known on the device, so every block derives the same plan from
// it: blocks [0, F) are whole, block F + k is split k % S of position block F + k / S.
struct TailPlan {
    int64_t whole;  // F: position blocks that run unsplit
    int64_t tail;   // position blocks of the last round
    int splits;     // S
};
__device__ __forceinline__ TailPlan tail_plan(int64_t n_xb, int slots)
{
    TailPlan p;
    p.whole = (n_xb / slots) * slots;
    p.tail = n_xb - p.whole;
    p.splits = 1;
    if (p.tail > 0 && p.tail * 2 <= slots) {
        const int s = (int)(slots / p.tail);
        p.splits = s < kTailMaxSplits ? s : kTailMaxSplits;
    }
    if (p.splits == 1) {  // nothing to gain: every block whole
        p.whole = n_xb;
        p.tail = 0;
    }
    return p;
}

template <int D, int MODE, int BY, int NW, int XG, int NBUF, int DS, bool FILTER = false>
__device__ __forceinline__ void tile_body(const TileArgs a, const int64_t block_id, uint16_t *const buf0, uint16_t *const buf1,
                                          uint16_t *const buf2, uint16_t *const buf3, float *const epi_own)
{
    constexpr bool BWD_MODE = (MODE != MODE_FWD);
    // The pipelined sub-tile loop alternates between two register sets; above d = 128 only the forward pass with one
    // group of stationary rows has the registers for it (the operands of a whole sub-tile are d/4 registers).
    constexpr bool SWP = (BY % 64 == 0) && (D <= 128 || (MODE == MODE_FWD && XG == 1));
    constexpr int KK = D / 16;             // k-steps of the score product
    constexpr int MB = D / 32;             // 32-row output blocks of the second product
    constexpr int CPR = D / 8;             // 16-byte chunks per row
    constexpr int SM = (CPR == 8) ? 7 : 15;  // chunk-index bits that the LDS swizzle permutes
    constexpr int NA = (KK < (SM + 1) / 2) ? KK : (SM + 1) / 2;  // distinct swizzled offsets of the operand reads
    constexpr int NT = (MB < (SM + 1) / 4) ? MB : (SM + 1) / 4;  // ... and of the transpose reads
    constexpr int XPB = (NW / DS) * XG * 32;  // stationary rows per block
    constexpr int MBH = MB / DS;           // output blocks of the second product that this wavefront accumulates
    static_assert(DS == 1 || (MODE != MODE_FWD && DS == 2 && NW % 2 == 0 && MBH % 4 == 0), "column split: backward passes, two ways, whole swizzle periods");
    constexpr int TILE = BY * D;           // elements per LDS tile
    constexpr int LOADS = BY * CPR / 64;   // 1-KiB direct-to-LDS load instructions per tile
    static_assert(LOADS % NW == 0, "tile loads must split evenly over the wavefronts");
    constexpr int LPW = LOADS / NW;
    static_assert(NBUF == 0 || (NBUF >= 2 && NBUF <= 4), "ring of 2 to 4 buffers, or 0 for the rolled form");
    constexpr int PF = (NBUF == 0) ? 1 : NBUF - 1;  // prefetch distance in tiles
    constexpr int NB = (NBUF == 0) ? 2 : NBUF;
    // A buffer holds the rows of a tile, (dE) the 2 x BY coefficient constants of its rows, and the row numbers of the
    // tile PF places further on, which ride along so that no load in the main loop returns into registers: the
    // outstanding-load count of a wavefront is then made of whole groups of known size.
    constexpr int IDS = (BY < 64) ? 64 : BY;                 // row numbers are fetched 64 at a time
    constexpr int CONSTS = (MODE == MODE_DE) ? 2 * BY : 0;   // 32-bit words
    constexpr int OFF_C = TILE, OFF_I = TILE + 2 * CONSTS;   // offsets in 16-bit elements
    constexpr int BUF = ((TILE + 2 * CONSTS + 2 * IDS + 511) / 512) * 512;
    constexpr int CI = (2 * BY / 64 < 1) ? 1 : 2 * BY / 64;  // 256-byte load instructions that fetch the constants
    constexpr int NI = IDS / 64;                             // ... and the row numbers
    static_assert(CI <= NW && NI <= NW, "every wavefront issues exactly one instruction of each kind");
    // dE epilogue: one 32 x 33 float transpose buffer per wavefront and the row numbers of the block.  They reuse the
    // first two tile buffers where those are big enough (two wavefronts' worth per buffer), else get an array.
    constexpr bool EPI_IN_TILES = (MODE == MODE_DE) && (NW == 4) && (TILE * 2 >= 2 * 32 * 33 * 4 + XPB * 8);
    static_assert(NW % 2 == 0, "wavefronts pair up on the tile buffers");

    // buf0..buf3 are separate LDS arrays of the calling kernel: the compiler then sees that operand reads of one buffer
    // cannot touch the buffers that loads are in flight into, and does not wait for them; the single-array form
    // (NBUF = 0) keeps one copy of the loop body where registers are short.
    auto buf_at = [&](int i) -> uint16_t * {
        if (NBUF == 0) return buf0 + (i & 1) * BUF;
        return i == 0 ? buf0 : (i == 1 ? buf1 : (i == 2 ? buf2 : buf3));
    };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lo = lane & 31;
    const int hi = lane >> 5;
    const int xgrp = wave / DS;   // group(s) of stationary rows of this wavefront
    const int half = wave % DS;   // its share of the output columns

    if (MODE == MODE_DE && block_id < a.pos_blocks) {  // leading blocks: scatter of the correct items
        static_assert(NW * 64 >= kPosChunk, "the scatter role needs 256 threads");
        pos_scatter_block<D>(a, block_id, reinterpret_cast<uint64_t *>(buf0));
        return;
    }
    if (MODE == MODE_DE && a.scale_blocks > 0 && block_id >= a.scale_block0) {  // trailing blocks: dH = grad_loss * U
#pragma unroll
        for (int j = 0; j < kScaleChunks; ++j)
            dh_scale_chunk<D>(a, ((block_id - a.scale_block0) * kScaleChunks + j) * (NW * 64) + tid);
        return;
    }
    if (MODE == MODE_DH && block_id < a.pad_blocks) {  // leading blocks: dH rows of padded positions are zero
        const int64_t i = block_id * (NW * 64) + tid;
        if (i < a.N) {
            bool valid = (a.pos_mask == nullptr) || (a.pos_mask[i] != 0);
            if (valid && a.validate) {  // a position with a target out of range counts as padding
                const int32_t ti = a.tgt[i];
                valid = ti >= 0 && (int64_t)ti < a.V;
            }
            if (!valid) {
                if (a.dH_bf16) {
                    uint4 *row = reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.dH) + i * D);
#pragma unroll 4
                    for (int c = 0; c < D / 8; ++c) row[c] = make_uint4(0, 0, 0, 0);
                } else {
                    float4 *row = reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + i * D);
#pragma unroll 4
                    for (int c = 0; c < D / 4; ++c) row[c] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
        return;
    }
    const int64_t bid = block_id - (MODE == MODE_DE ? a.pos_blocks : (MODE == MODE_DH ? a.pad_blocks : 0));
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t n_x = (MODE == MODE_DE) ? a.n_cols : n_pos;
    const int64_t n_y = (MODE == MODE_DE) ? n_pos : a.n_cols;
    int split = (int)(bid % a.splits), splits = a.splits;
    int64_t xb = bid / a.splits;
    int64_t part_rows = a.N, part_x0 = 0;  // partial dH rows of split runs: rows per split, first position filed there
    if ((MODE == MODE_DH || MODE == MODE_FDH) && a.tail_slots > 0) {  // last-round split, planned from the device-side count (a.splits == 1)
        const TailPlan tp = tail_plan((n_x + XPB - 1) / XPB, a.tail_slots);
        if (bid >= tp.whole) {
            xb = tp.whole + (bid - tp.whole) / tp.splits;
            split = (int)((bid - tp.whole) % tp.splits);
            splits = tp.splits;
            part_rows = tp.tail * XPB;
            part_x0 = tp.whole * XPB;
            if (bid >= tp.whole + tp.tail * tp.splits) return;
        }
    }
    if (xb * XPB >= n_x) return;  // whole block past the end (the grid is sized for the unmasked N)

    const uint16_t *Xbase = (MODE == MODE_DE) ? a.E : a.H;
    const uint16_t *Ybase = (MODE == MODE_DE) ? a.H : a.E;

    // ---- stationary rows -> registers in B-operand layout: lane (lo, hi) holds X[x][kk*16 + hi*8 .. +8]
    int64_t xrow[XG];
    bool x_ok[XG];
    uint4 xr[XG][KK];
    float cx[XG];  // DH: -lse * log2(e) of the lane's position
#pragma unroll
    for (int g = 0; g < XG; ++g) {
        const int64_t x = xb * XPB + (xgrp * XG + g) * 32 + lo;
        x_ok[g] = x < n_x;
        xrow[g] = (MODE == MODE_DE) ? item_row(a, x_ok[g] ? x : 0) : pos_row(a, x_ok[g] ? x : 0);
        const uint16_t *xp = Xbase + xrow[g] * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) xr[g][kk] = *reinterpret_cast<const uint4 *>(xp + kk * 16 + hi * 8);
        cx[g] = 0.f;
        if (MODE == MODE_DH) {
            cx[g] = -a.lse_in[xrow[g]] * kLog2e;
            // The dE pass wants g * exp(o - lse) = g * 2^(o log2e - lse log2e) for every position it streams: the
            // offset and g are filed here under the compacted index, where that pass finds them in order.
            if (a.write_consts && split == 0 && hi == 0 && half == 0 && x_ok[g]) {
                const float gg = a.g ? a.g[xrow[g]] : 1.f;
                a.de_const[x] = __float_as_uint(cx[g]);
                a.de_const[a.N + x] = __float_as_uint(gg);
            }
        }
    }

    // ---- range of streamed tiles of this split
    const int64_t n_tiles = (n_y + BY - 1) / BY;
    const int64_t t_begin = n_tiles * split / splits;
    const int64_t t_end = n_tiles * (split + 1) / splits;

    f32x16 acc[XG][MODE == MODE_FWD ? 1 : MBH];
    if (MODE != MODE_FWD) {
#pragma unroll
        for (int g = 0; g < XG; ++g)
#pragma unroll
            for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[g][mb][q] = 0.f;
    }
    float run_m[XG], run_s[XG];  // FWD: base-2 running max and sum of this lane's half of the candidates
#pragma unroll
    for (int g = 0; g < XG; ++g) {
        run_m[g] = -INFINITY;
        run_s[g] = 0.f;
    }

    // ---- streamed tiles: global memory -> LDS without passing through registers.  One instruction moves 1 KiB:
    //      lane l of the wavefront writes 16 bytes at (wave-uniform base) + 16 l, so the lane that owns LDS slot
    //      (row r, physical chunk pc) fetches the logical chunk pc ^ swz(r) of that row.
    const int32_t *const ind = (MODE == MODE_DE) ? a.idx : a.neg;  // streamed index -> row; nullptr = identity
    const int group_extras = (MODE == MODE_DE ? 1 : 0) + (ind ? 1 : 0);  // instructions per group beyond LPW
    auto checked_row = [&](int32_t id) -> int32_t {
        if (MODE != MODE_DE && a.validate && (id < 0 || (int64_t)id >= a.V)) id = 0;  // flagged by the preparation kernel
        return id;
    };
    // Row numbers of a tile's rows, as each lane needs them for its LPW load instructions: straight from global memory
    // (prologue), or from the copy that an earlier load group left in LDS.
    // rows[LPW] is the row whose constant (dE pass) this lane's constant load fetches.
    constexpr int NR = LPW + 1;
    constexpr bool GSEP = (MODE == MODE_DE) && D <= 128;  // only the fused backward launch (hidden sizes up to 128) uses it
    auto const_row_slot = [&]() -> int { return ((wave % CI) * 64 + lane) % BY; };
    auto rows_from_global = [&](int64_t t, int32_t (&rows)[NR]) {
        rows[LPW] = 0;
        if (GSEP && a.g_separate && !a.g_stream_off) {
            int64_t y = t * BY + const_row_slot();
            if (y >= n_y) y = n_y - 1;
            rows[LPW] = ind ? ind[y] : (int32_t)y;
        }
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = ((wave + i * NW) * 64 + lane) / CPR;
            int64_t y = t * BY + r;
            if (y >= n_y) y = n_y - 1;  // rows past the end repeat the last row (finite data); they are masked below
            rows[i] = ind ? checked_row(ind[y]) : (int32_t)y;
        }
    };
    // Everything per lane in here is recomputed from the thread number at every step: kept across the loop, these
    // values are the first that the register allocator spills, and a reload from scratch memory waits, as the counter of
    // vector-memory operations runs in order, for every tile load in flight.
    auto rows_from_lds = [&](int64_t t, const uint16_t *holder, int32_t (&rows)[NR]) {
        const int32_t *ids = reinterpret_cast<const int32_t *>(holder + OFF_I);
        const uint32_t y0 = (uint32_t)(t * BY), y_last = (uint32_t)(n_y - 1);  // t * BY < n_y < 2^31
        uint32_t me = (uint32_t)tid;
        asm volatile("" : "+v"(me));
        const uint32_t r0 = me / CPR;  // CPR divides 64: instruction i of this lane fetches row r0 + i * (NW * 64 / CPR)
        rows[LPW] = 0;
        if (GSEP && a.g_separate && !a.g_stream_off) {
            const uint32_t slot = (((me >> 6) % CI) * 64 + (me & 63)) % BY;  // const_row_slot()
            const uint32_t y = y0 + slot;
            rows[LPW] = ind ? ids[slot] : (int32_t)(y < y_last ? y : y_last);
        }
        if (ind) {
#pragma unroll
            for (int i = 0; i < LPW; ++i) rows[i] = checked_row(ids[r0 + i * (NW * 64 / CPR)]);
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const uint32_t y = y0 + r0 + (uint32_t)(i * (NW * 64 / CPR));
                rows[i] = (int32_t)(y < y_last ? y : y_last);
            }
        }
    };
    // One load group: the rows of tile t, (dE) the constants of its rows, and the row numbers of tile t + PF.
    // Byte offset inside a streamed row of the chunk that instruction i of this lane fetches: the same for every tile.
    // A load then costs one shift-add per lane on top of the row number, as long as the streamed table is below
    // 4 GiB (32-bit offsets from a uniform base); larger tables take 64-bit addresses.
    uint32_t chunk_ofs[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int L = (wave + i * NW) * 64 + lane;
        const int r = L / CPR, pc = L % CPR;
        chunk_ofs[i] = (uint32_t)(((pc & ~SM) | ((pc & SM) ^ swz<CPR>(r))) * 16);
    }
    const bool small_table = (uint64_t)((MODE == MODE_DE) ? a.N : a.V) * (uint64_t)(D * 2) <= 0xffffffffull;
    const char *const Ybytes = reinterpret_cast<const char *>(Ybase);
    const uint32_t last_y = (uint32_t)(n_y - 1);
    // The destination reaches the load instructions as a bare LDS offset that the optimiser cannot trace back to its
    // array.  Otherwise the compiler, which does not see the counted waits of the ring (they are inline assembly),
    // protects the one buffer that is filled and read within one trip of the unrolled loop with a wait for ALL loads in
    // flight, placed right after the group of the next tile has been issued: the load latency of every NBUF-th tile
    // was then exposed in full.  That a tile has landed before it is read is the business of wait_for_next() and the
    // barrier behind it, for every buffer alike.
    auto issue_group = [&](int64_t t, const int32_t (&rows)[NR], uint16_t *dst_generic) {
        uint32_t dst_lds = (uint32_t)(uintptr_t)(lds_ptr)dst_generic;
        asm volatile("" : "+s"(dst_lds));
        uint16_t __attribute__((address_space(3))) *dst = (uint16_t __attribute__((address_space(3))) *)(uintptr_t)dst_lds;
        if (small_table) {
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const uint32_t ofs = (uint32_t)rows[i] * (uint32_t)(D * 2) + chunk_ofs[i];
                __builtin_amdgcn_global_load_lds((global_cptr)(Ybytes + ofs), (lds_ptr)(dst + (wave + i * NW) * 512), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                uint32_t co = chunk_ofs[i];
                asm volatile("" : "+v"(co));  // keeps the per-lane sum Ybytes + chunk_ofs from being carried (and spilled) as a 64-bit pair
                const char *src = Ybytes + ((int64_t)rows[i] * (D * 2) + co);
                __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)(dst + (wave + i * NW) * 512), 16, 0, 0);
            }
        }
        if (MODE == MODE_DE) {  // wavefronts beyond CI repeat a load (same data, same place): group sizes stay uniform
            const int inst = wave % CI;
            const int e = inst * 64 + lane;
            uint32_t y = (uint32_t)(t * BY) + (uint32_t)(e % BY);  // t * BY < n_y < 2^31
            if (y > last_y) y = last_y;
            const uint32_t *src = a.de_const + (int64_t)(e / BY) * a.N + y;
            // upstream gradient straight from the caller's array, by row number, where the forward pass left the rest
            if (GSEP && a.g_separate && !a.g_stream_off && e / BY == 1) src = reinterpret_cast<const uint32_t *>(a.g) + rows[LPW];
            __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)(dst + OFF_C + inst * 128), 4, 0, 0);
        }
        if (ind) {
            const int inst = wave % NI;
            const int64_t t_ids = (t + PF) * BY < n_y ? (t + PF) * BY : n_y - 1;  // uniform
            uint32_t y = (uint32_t)t_ids + (uint32_t)(inst * 64 + lane);
            if (y > last_y) y = last_y;
            __builtin_amdgcn_global_load_lds((global_cptr)(ind + y), (lds_ptr)(dst + OFF_I + inst * 128), 4, 0, 0);
        }
    };

    // per-lane pieces of the swizzled LDS addresses (elements)
    // Every swizzled offset is one of two per-lane bases XORed with a compile-time constant: the chunk index of an
    // operand read is (kk*2) ^ hi ^ swz(row), that of a transpose read (mb*4) ^ (cb*2 + tb/2) ^ swz(row), and the
    // row part of the offset has no bits in common with the chunk part.  Where registers are short (LEAN) the XOR is
    // redone at every read instead of being kept in a register per constant.
    constexpr bool LEAN = (D >= 256 && DS == 1 && (BWD_MODE || XG == 2)) || (D == 128 && BWD_MODE);
    const int a_base = lo * D + ((hi ^ swz<CPR>(lo)) * 8);  // operand reads of the score product: row lo, chunk kk*2 + hi
    const int j16 = lane & 15, ta = j16 >> 2, tb = j16 & 3, cb = (lane >> 4) & 1;
    // transpose reads of the second product: rows hi*4 + ta and 8 below (whose swizzle differs in bit 1), chunk
    // mb*4 + cb*2 + tb/2, four elements per lane
    const int t_row = hi * 4 + ta;
    const int t_base0 = t_row * D + (((cb * 2 + (tb >> 1)) ^ swz<CPR>(t_row)) * 8) + (tb & 1) * 4;
    const int t_base1 = (t_base0 ^ 16) + 8 * D;
    // Address of element (base ^ bits) + extra behind p.  LEAN: the XOR is done on byte offsets (no shift between it and
    // the read) by an instruction the optimiser cannot hoist out of the loop.
    auto lds_at = [&](const uint16_t *p, int base, int bits, int extra) -> const uint16_t * {
        if (LEAN) {
            int r;
            asm volatile("v_xor_b32 %0, %1, %2" : "=v"(r) : "s"(bits * 2), "v"(base * 2));
            return reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(p) + r) + extra;
        }
        return p + (base ^ bits) + extra;
    };

    constexpr int NSB = BY / 32;
    constexpr bool BWD = (MODE != MODE_FWD);
    typedef uint32_t gp_t[XG][8];  // probabilities / coefficients of one sub-tile as bf16 pairs: B operand of the second product

    // ---- the four pieces of a sub-tile: operand reads, score product, softmax arithmetic, second product
    auto load_ops = [&](const uint16_t *tile, int sb, uint4 (&op)[KK]) {
        const uint16_t *arow = tile + sb * 32 * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            op[kk] = *reinterpret_cast<const uint4 *>(lds_at(arow, a_base, ((kk * 2) & SM) * 8, (kk / NA) * (NA * 16)));
    };
    auto mfma_scores = [&](const uint4 (&op)[KK], f32x16 (&sv)[XG]) {
#pragma unroll
        for (int g = 0; g < XG; ++g)
#pragma unroll
            for (int q = 0; q < 16; ++q) sv[g][q] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int g = 0; g < XG; ++g)
                sv[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(op[kk]), as_bf16x8(xr[g][kk]), sv[g], 0, 0, 0);
    };
    // accumulator register q of lane (lo, hi) holds streamed row y = sb*32 + (q/4)*8 + hi*4 + q%4
    auto softmax = [&](const uint16_t *tile, int sb, f32x16 (&sv)[XG], gp_t &gp, int rows_here, auto ragged_tag, bool &kept,
                       auto max_tag) {
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        constexpr bool LAZY = decltype(max_tag)::lazy;
        const int rem = rows_here - sb * 32 - hi * 4;  // register q is a real row iff (q/4)*8 + q%4 < rem
        if (MODE == MODE_FWD && LAZY) {
            // Any reference keeps the sum of exponentials exact as long as nothing overflows; the one in hand saves the
            // maximum chain and the rescaling (a fifth of the vector instructions of the forward pass).
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                const float ref = -run_m[g];
                float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 16; ++q) part[q & 3] += __builtin_amdgcn_exp2f(fmaf(sv[g][q], kLog2e, ref));
                run_s[g] += (part[0] + part[1]) + (part[2] + part[3]);
            }
        } else if (MODE == MODE_FWD) {
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                if (RAGGED) {  // rows past the end do not take part
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if ((q / 4) * 8 + (q % 4) >= rem) sv[g][q] = -INFINITY;
                }
                // The compiler pads matrix-instruction results with the wait states their first vector reader needs,
                // but it does not look inside inline assembly: the first reader of this score tile is therefore a
                // plain multiply, and the max3 chain is tied behind it.
                const float last = sv[g][15] * kLog2e;
                float tm = max3_after(last, sv[g][0], sv[g][1], sv[g][2]);
#pragma unroll
                for (int q = 3; q < 15; q += 2) tm = max3(tm, sv[g][q], sv[g][q + 1]);
                const float mn = max3(run_m[g], tm * kLog2e, last);
                if (!RAGGED || mn > -INFINITY) {  // a full sub-tile always has a finite maximum
                    float part[4] = {0.f, 0.f, 0.f, 0.f};  // four short chains instead of one long one
#pragma unroll
                    for (int q = 0; q < 16; ++q) part[q & 3] += __builtin_amdgcn_exp2f(fmaf(sv[g][q], kLog2e, -mn));
                    run_s[g] = run_s[g] * __builtin_amdgcn_exp2f(run_m[g] - mn) + ((part[0] + part[1]) + (part[2] + part[3]));
                    run_m[g] = mn;
                }
            }
        } else if (MODE == MODE_FDH) {
            // One pass for the forward sum and for the probabilities of the second product: 2^(o log2e - ref) against the
            // block's reference (see the FDH notes at the streaming loop); the sum is kept in fp32 from the unrounded
            // values, the second product takes them rounded to bf16, and the epilogue divides by the sum.
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                const float ref = -run_m[g];
                float v[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) v[q] = __builtin_amdgcn_exp2f(fmaf(sv[g][q], kLog2e, ref));
                if (RAGGED) {
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if ((q / 4) * 8 + (q % 4) >= rem) v[q] = 0.f;
                }
                float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 16; ++q) part[q & 3] += v[q];
                run_s[g] += (part[0] + part[1]) + (part[2] + part[3]);
#pragma unroll
                for (int q = 0; q < 16; q += 2) gp[g][q / 2] = pack2(v[q], v[q + 1]);
            }
        } else {
            const float *yc = reinterpret_cast<const float *>(tile + OFF_C);
            const float *yg = reinterpret_cast<const float *>(tile + OFF_C) + BY;
            if constexpr (FILTER) {
                // Gradient filtering: this wavefront's 32 stationary rows by the 32 streamed rows of the sub-tile are one
                // block of the softmax matrix (both passes cut it the same way: positions by 32 in compacted order,
                // items by 32 in id order).  Its probabilities are 2^a with a = o log2e - lse log2e; if none reaches the
                // threshold the block contributes nothing, and neither exponentials nor the second product are spent.
                kept = false;
#pragma unroll
                for (int g = 0; g < XG; ++g) {
                    float lg[16];
                    float4 gy[4];
                    if (MODE == MODE_DH) {
#pragma unroll
                        for (int q = 0; q < 16; ++q) lg[q] = fmaf(sv[g][q], kLog2e, cx[g]);
                    } else {
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq) {
                            const float4 cy = *reinterpret_cast<const float4 *>(&yc[sb * 32 + qq * 8 + hi * 4]);
                            gy[qq] = *reinterpret_cast<const float4 *>(&yg[sb * 32 + qq * 8 + hi * 4]);
                            lg[qq * 4 + 0] = fmaf(sv[g][qq * 4 + 0], kLog2e, cy.x);
                            lg[qq * 4 + 1] = fmaf(sv[g][qq * 4 + 1], kLog2e, cy.y);
                            lg[qq * 4 + 2] = fmaf(sv[g][qq * 4 + 2], kLog2e, cy.z);
                            lg[qq * 4 + 3] = fmaf(sv[g][qq * 4 + 3], kLog2e, cy.w);
                        }
                    }
                    if (RAGGED) {
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            if ((q / 4) * 8 + (q % 4) >= rem) lg[q] = -INFINITY;
                    }
                    float big = max3(lg[0], lg[1], lg[2]);
#pragma unroll
                    for (int q = 3; q < 15; q += 2) big = max3(big, lg[q], lg[q + 1]);
                    big = fmaxf(big, lg[15]);
                    // stationary rows past the end hold a copy of row 0: they must not keep a block alive
                    const bool keep_g = __any(x_ok[g] && big >= a.filter_log2);
                    if (keep_g) {
#pragma unroll
                        for (int q = 0; q < 16; q += 2) {
                            float v0 = __builtin_amdgcn_exp2f(lg[q]), v1 = __builtin_amdgcn_exp2f(lg[q + 1]);
                            if (MODE == MODE_DE) {
                                const float4 &gq = gy[q / 4];
                                v0 *= (q % 4 == 0) ? gq.x : gq.z;
                                v1 *= (q % 4 == 0) ? gq.y : gq.w;
                            }
                            gp[g][q / 2] = pack2(v0, v1);
                        }
                        kept = true;
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) gp[g][q] = 0u;
                    }
                }
                return;
            }
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                float v[16];
                if (MODE == MODE_DH) {
#pragma unroll
                    for (int q = 0; q < 16; ++q) v[q] = __builtin_amdgcn_exp2f(fmaf(sv[g][q], kLog2e, cx[g]));
                } else {
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const float4 cy = *reinterpret_cast<const float4 *>(&yc[sb * 32 + qq * 8 + hi * 4]);
                        const float4 gy = *reinterpret_cast<const float4 *>(&yg[sb * 32 + qq * 8 + hi * 4]);
                        v[qq * 4 + 0] = gy.x * __builtin_amdgcn_exp2f(fmaf(sv[g][qq * 4 + 0], kLog2e, cy.x));
                        v[qq * 4 + 1] = gy.y * __builtin_amdgcn_exp2f(fmaf(sv[g][qq * 4 + 1], kLog2e, cy.y));
                        v[qq * 4 + 2] = gy.z * __builtin_amdgcn_exp2f(fmaf(sv[g][qq * 4 + 2], kLog2e, cy.z));
                        v[qq * 4 + 3] = gy.w * __builtin_amdgcn_exp2f(fmaf(sv[g][qq * 4 + 3], kLog2e, cy.w));
                    }
                }
                if (RAGGED) {
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if ((q / 4) * 8 + (q % 4) >= rem) v[q] = 0.f;
                }
#pragma unroll
                for (int q = 0; q < 16; q += 2) gp[g][q / 2] = pack2(v[q], v[q + 1]);
            }
        }
    };
    // out^T[t, x] += sum_y Y[y, t] * G^T[y, x]; the A operand is read transposed from the row-major tile
    auto load_tr = [&](const uint16_t *tile, int sb, s16x8 (&tr)[2][MBH]) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const uint16_t *tbase = tile + (sb * 32 + k2 * 16) * D + half * (MBH * 32);  // this wavefront's columns
#pragma unroll
            for (int mb = 0; mb < MBH; ++mb) {
                const int col = (mb / NT) * (NT * 32);
                const s16x4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(lds_at(tbase, t_base0, ((mb * 4) & SM) * 8, col)));
                const s16x4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(lds_at(tbase, t_base1, ((mb * 4) & SM) * 8, col)));
                tr[k2][mb] = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    auto second = [&](const s16x8 (&tr)[2][MBH], const gp_t &gp) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int mb = 0; mb < MBH; ++mb) {
                bf16x8 av;
                __builtin_memcpy(&av, &tr[k2][mb], 16);
#pragma unroll
                for (int g = 0; g < XG; ++g) {
                    const uint4 bv = make_uint4(gp[g][k2 * 4 + 0], gp[g][k2 * 4 + 1], gp[g][k2 * 4 + 2], gp[g][k2 * 4 + 3]);
                    acc[g][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, as_bf16x8(bv), acc[g][mb], 0, 0, 0);
                }
            }
    };

    // A tile is NSB sub-tiles of 32 streamed rows.  Matrix and vector work per sub-tile are about equal at d = 64
    // (measured 122 ns against 120 ns per SIMD); the matrix pipe is asynchronous, but a wavefront issues in order,
    // and neither two nor three wavefronts per SIMD overlap the two units on their own.  So the sub-tile loop is
    // unrolled and software-pipelined inside the wavefront: while the softmax arithmetic of sub-tile k runs, the
    // matrix pipe works through the second product of sub-tile k - 1 and the score product of sub-tile k + 1, one
    // matrix instruction per slice of vector work, and the LDS operands of a product are requested a phase ahead of
    // it.  The compiler's scheduler is told that order explicitly; left alone it issues the matrix instructions of a
    // whole tile first and the vector work after them.
    // The short last tile of the streamed range takes a separate copy of the code (RAGGED), so that full tiles have
    // no branch or select in this loop.
    constexpr int NM_S = KK * XG;                 // matrix instructions of a score product
    constexpr int NM_P = BWD ? 2 * MBH * XG : 0;  // ... of a second product
    constexpr int N_TR = 4 * MBH;                 // transpose reads of a second product
    constexpr int VALU_C = XG * (MODE == MODE_FWD ? 56 : (MODE == MODE_DH ? 42 : 58));  // vector instructions of a softmax (FDH: 58)
    auto process_tile = [&](int64_t t, const uint16_t *tile, auto ragged_tag, auto max_tag) {
        // rows of this tile that exist; only the last tile of the streamed range can be short
        const int rows_here = (n_y - t * BY < BY) ? (int)(n_y - t * BY) : BY;
        if constexpr (SWP) {
            static_assert(!SWP || NSB % 2 == 0, "the pipelined loop alternates between two register sets");
            uint4 op[2][KK];
            f32x16 sv[2][XG];
            gp_t gp[2];
            s16x8 tr[2][MBH];
            bool kept[2] = {true, true};  // gradient filtering: whether the sub-tile of either register set survived
            // Forward: operands two sub-tiles ahead (nothing else covers their latency).  Backward: one ahead, and the
            // second product of the previous sub-tile goes to the matrix pipe before the score product that needs them.
            constexpr int OPD = (BWD || D > 128) ? 1 : 2;
            load_ops(tile, 0, op[0]);
            if (OPD == 2 && NSB > 1) load_ops(tile, 1, op[1]);
            mfma_scores(op[0], sv[0]);
            __builtin_amdgcn_sched_group_barrier(0x100, OPD * KK, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, NM_S, 0);
#pragma unroll
            for (int k = 0; k < NSB; ++k) {
                const int c = k & 1, n = c ^ 1;
                const int opn = (OPD == 2) ? n : 0, opl = (OPD == 2) ? c : 0;  // set S(k+1) reads / set loaded now
                if (k + OPD < NSB) load_ops(tile, k + OPD, op[opl]);
                if (BWD && k > 0 && kept[n]) second(tr, gp[n]);
                if (k + 1 < NSB) mfma_scores(op[opn], sv[n]);
                softmax(tile, k, sv[c], gp[c], rows_here, ragged_tag, kept[c], max_tag);
                if (BWD && kept[c]) load_tr(tile, k, tr);
                // ---- issue order of this phase
                const int n_mfma = ((BWD && k > 0) ? NM_P : 0) + (k + 1 < NSB ? NM_S : 0);
                if (k + OPD < NSB) __builtin_amdgcn_sched_group_barrier(0x100, KK, 0);
                if (n_mfma == NM_P + NM_S) {
#pragma unroll
                    for (int i = 0; i < NM_P + NM_S; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, (VALU_C + NM_P + NM_S - 1) / (NM_P + NM_S), 0);
                    }
                } else if (n_mfma == NM_S) {
#pragma unroll
                    for (int i = 0; i < NM_S; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, (VALU_C + NM_S - 1) / NM_S, 0);
                    }
                } else if (n_mfma > 0) {
#pragma unroll
                    for (int i = 0; i < NM_P; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, (VALU_C + (NM_P > 0 ? NM_P : 1) - 1) / (NM_P > 0 ? NM_P : 1), 0);
                    }
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x002, VALU_C, 0);
                }
                if (BWD) __builtin_amdgcn_sched_group_barrier(0x100, N_TR, 0);
            }
            if (BWD && kept[(NSB - 1) & 1]) {
                second(tr, gp[(NSB - 1) & 1]);
                __builtin_amdgcn_sched_group_barrier(0x008, NM_P, 0);
            }
        } else {
            // Large hidden sizes, backward passes: no room for a second sub-tile in flight, the other wavefront of the
            // SIMD fills the gaps.  What must not happen is one LDS read per matrix instruction with the read issued just ahead of
            // it, as the compiler orders them: LDS latency is several times the 32 cycles of a matrix instruction.
            // Operands are therefore read in batches of four into two alternating register sets, and every batch is
            // requested one batch of matrix instructions ahead of its use.
            constexpr int BS = (DS == 1 && BWD) ? 2 : 4;  // operands per batch: two where all output columns are held
            // operand batches in flight: three in the dH pass (measured 2 % faster at d = 256), two elsewhere (in the dE
            // pass the third costs spilled registers and 7 %)
            constexpr int RD = (DS == 1 && (MODE == MODE_DH || MODE == MODE_FDH)) ? 3 : 2;
            constexpr int NB_S = KK / BS;         // batches of the score product
            constexpr int NB_P = 2 * MBH / BS;    // batches of the second product
            static_assert(KK % BS == 0 && MBH % BS == 0, "whole operand batches");
#pragma unroll 1
            for (int sb = 0; sb < NSB; ++sb) {
                f32x16 sv[XG];
                gp_t gp;
                uint4 ob[RD][BS];
                const uint16_t *arow = tile + sb * 32 * D;
                // PAIRED (register-lean addressing): the two reads of a batch are the ones whose swizzled offsets agree
                // (pieces kk and kk + NA; output blocks mb and mb + NT), so that one XOR serves both and the rest of the
                // address is an immediate: a third of the vector instructions of a step were such XORs.
                constexpr bool PAIRED = LEAN && BS == 2 && KK == 2 * NA && MBH == 2 * NT;
                auto s_piece = [&](int b, int i) { return PAIRED ? b + i * NA : b * BS + i; };
                auto p_block = [&](int b, int i) { return PAIRED ? (b % (MBH / BS)) + i * NT : (b % (MBH / BS)) * BS + i; };
                auto read_batch = [&](int b, uint4 (&dst)[BS]) {
                    if constexpr (PAIRED) {
                        const uint16_t *q = lds_at(arow, a_base, ((b * 2) & SM) * 8, 0);
                        dst[0] = *reinterpret_cast<const uint4 *>(q);
                        dst[1] = *reinterpret_cast<const uint4 *>(q + NA * 16);
                        return;
                    }
#pragma unroll
                    for (int i = 0; i < BS; ++i) {
                        const int kk = b * BS + i;
                        dst[i] = *reinterpret_cast<const uint4 *>(lds_at(arow, a_base, ((kk * 2) & SM) * 8, (kk / NA) * (NA * 16)));
                    }
                };
#pragma unroll
                for (int g = 0; g < XG; ++g)
#pragma unroll
                    for (int q = 0; q < 16; ++q) sv[g][q] = 0.f;
#pragma unroll
                for (int b = 0; b < RD && b < NB_S; ++b) read_batch(b, ob[b]);
#pragma unroll
                for (int b = 0; b < NB_S; ++b) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < BS; ++i)
#pragma unroll
                        for (int g = 0; g < XG; ++g)
                            sv[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ob[b % RD][i]), as_bf16x8(xr[g][s_piece(b, i)]), sv[g], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (b + RD < NB_S) read_batch(b + RD, ob[b % RD]);
                }
                if (BWD) {
                    // transpose reads of the first two batches go out before the softmax arithmetic and land under it
                    s16x8 tb[RD][BS];
                    auto read_tr_batch = [&](int b, s16x8 (&dst)[BS]) {
                        const int k2 = b / (MBH / BS);
                        const uint16_t *tbase = tile + (sb * 32 + k2 * 16) * D + half * (MBH * 32);
                        if constexpr (PAIRED) {
                            const int mb0 = b % (MBH / BS);
                            const uint16_t *q0 = lds_at(tbase, t_base0, ((mb0 * 4) & SM) * 8, 0);
                            const uint16_t *q1 = lds_at(tbase, t_base1, ((mb0 * 4) & SM) * 8, 0);
#pragma unroll
                            for (int i = 0; i < BS; ++i) {
                                const s16x4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(q0 + i * (NT * 32)));
                                const s16x4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(q1 + i * (NT * 32)));
                                dst[i] = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
                            }
                            return;
                        }
#pragma unroll
                        for (int i = 0; i < BS; ++i) {
                            const int mb = (b % (MBH / BS)) * BS + i;
                            const int col = (mb / NT) * (NT * 32);
                            const s16x4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(lds_at(tbase, t_base0, ((mb * 4) & SM) * 8, col)));
                            const s16x4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(lds_at(tbase, t_base1, ((mb * 4) & SM) * 8, col)));
                            dst[i] = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
                        }
                    };
                    bool kept = true;
                    if (FILTER) {  // the reads wait for the verdict on the block
                        softmax(tile, sb, sv, gp, rows_here, ragged_tag, kept, max_tag);
                        if (!kept) continue;
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int b = 0; b < RD && b < NB_P; ++b) read_tr_batch(b, tb[b]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (!FILTER) softmax(tile, sb, sv, gp, rows_here, ragged_tag, kept, max_tag);
#pragma unroll
                    for (int b = 0; b < NB_P; ++b) {
                        __builtin_amdgcn_sched_barrier(0);
                        const int k2 = b / (MBH / BS);
#pragma unroll
                        for (int i = 0; i < BS; ++i) {
                            const int mb = p_block(b, i);
                            bf16x8 av;
                            __builtin_memcpy(&av, &tb[b % RD][i], 16);
#pragma unroll
                            for (int g = 0; g < XG; ++g) {
                                const uint4 bv = make_uint4(gp[g][k2 * 4 + 0], gp[g][k2 * 4 + 1], gp[g][k2 * 4 + 2], gp[g][k2 * 4 + 3]);
                                acc[g][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, as_bf16x8(bv), acc[g][mb], 0, 0, 0);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (b + RD < NB_P) read_tr_batch(b + RD, tb[b % RD]);
                    }
                } else {
                    bool kept = true;
                    softmax(tile, sb, sv, gp, rows_here, ragged_tag, kept, max_tag);
                }
            }
        }
    };

    // The last tile of the whole streamed range may be short; it is left out of the main loop and handled after it.
    const bool tail_ragged = (n_y % BY) != 0 && t_end == n_tiles && t_end > t_begin;
    const int64_t t_stop = tail_ragged ? t_end - 1 : t_end;  // tiles [t_begin, t_stop) are full

    // Step t: start the group of tile t + PF (into the buffer that tile t - 1 has just left), work on tile t, then
    // wait until tile t + 1 has landed: the groups issued after it are those of tiles t + 2 .. t + PF.
    auto wait_for_next = [&](int64_t t) {
        int younger = 0;
#pragma unroll
        for (int k = 2; k <= PF; ++k) younger += (t + k < t_end) ? 1 : 0;
        wait_all_but<LPW>(younger, group_extras);
    };
    // Keeps the arithmetic of a tile in front of the wait that follows it: without a use at this point the compiler
    // sinks the whole softmax update below the wait, into the next step, where no matrix work is left to overlap it.
    auto pin_results = [&]() {
        if (MODE == MODE_FWD) {
#pragma unroll
            for (int g = 0; g < XG; ++g) asm volatile("" : "+v"(run_m[g]), "+v"(run_s[g]));
        }
        if (MODE == MODE_FDH) {
#pragma unroll
            for (int g = 0; g < XG; ++g) asm volatile("" : "+v"(run_s[g]));
        }
    };
    // ---- FDH: forward sum and hidden-state gradient in one pass (an online softmax, Alg. 1, carried through Eq. 6 left).
    // The probabilities of the second product are taken against a reference m per position instead of the final
    // log-sum-exp: acc = sum_j 2^(o_j log2e - m) E_j, run_s = sum_j 2^(o_j log2e - m), and the epilogue divides.  Any m
    // gives the same result as long as nothing leaves the float range, so the fast attempt takes m = the largest score
    // among the first 32 candidates of the block's range and never looks at a maximum again (no maximum chain, no
    // rescaling, no branch inside the software-pipelined loop).  Scores that outgrow that reference by more than about
    // 69 nats push a sum beyond 1e30: the wavefront that sees it raises a flag in LDS, every wavefront of the block reads
    // the flag of the previous tile during a step (two flags, by tile parity, so that all of them read the same
    // value), and the block starts over in the exact form: the largest score of every tile is taken first (a score
    // product of its own), sums and accumulators are rescaled when it grows, and no exponent is ever positive.
    int *const over_flag = reinterpret_cast<int *>(epi_own);
    auto tile_max = [&](const uint16_t *tile, int nsub, int rows_here, float (&tmax)[XG]) {
#pragma unroll
        for (int g = 0; g < XG; ++g) tmax[g] = -INFINITY;
#pragma unroll 1
        for (int sb = 0; sb < nsub; ++sb) {
            f32x16 sv[XG];
#pragma unroll
            for (int g = 0; g < XG; ++g)
#pragma unroll
                for (int q = 0; q < 16; ++q) sv[g][q] = 0.f;
            const uint16_t *arow = tile + sb * 32 * D;
#pragma unroll
            for (int kk = 0; kk < KK; kk += 2) {  // two operands at a time: registers are short at large hidden sizes
                const uint4 o0 = *reinterpret_cast<const uint4 *>(lds_at(arow, a_base, ((kk * 2) & SM) * 8, (kk / NA) * (NA * 16)));
                const uint4 o1 = *reinterpret_cast<const uint4 *>(lds_at(arow, a_base, (((kk + 1) * 2) & SM) * 8, ((kk + 1) / NA) * (NA * 16)));
#pragma unroll
                for (int g = 0; g < XG; ++g) {
                    sv[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(o0), as_bf16x8(xr[g][kk]), sv[g], 0, 0, 0);
                    sv[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(o1), as_bf16x8(xr[g][kk + 1]), sv[g], 0, 0, 0);
                }
            }
            const int rem = rows_here - sb * 32 - hi * 4;
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                float tm = -INFINITY;
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if ((q / 4) * 8 + (q % 4) < rem) tm = fmaxf(tm, sv[g][q]);
                tmax[g] = fmaxf(tmax[g], tm * kLog2e);
            }
        }
#pragma unroll
        for (int g = 0; g < XG; ++g) tmax[g] = fmaxf(tmax[g], __shfl_xor(tmax[g], 32, 64));  // both halves of a position agree
    };
    // Exact form: bring the reference up to the largest score of the tile at hand before its exponentials are taken.
    auto raise_reference = [&](const uint16_t *tile, int rows_here) {
        float tmax[XG];
        tile_max(tile, NSB, rows_here, tmax);
        bool grow = false;
#pragma unroll
        for (int g = 0; g < XG; ++g) grow |= tmax[g] > run_m[g];
        if (__any(grow)) {
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                const float mn = fmaxf(run_m[g], tmax[g]);
                const float sc = (mn == run_m[g]) ? 1.f : __builtin_amdgcn_exp2f(run_m[g] - mn);  // first tile: 2^-inf = 0
                run_m[g] = mn;
                run_s[g] *= sc;
#pragma unroll
                for (int mb = 0; mb < (MODE == MODE_FWD ? 1 : MBH); ++mb)
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[g][mb][q] *= sc;
            }
        }
    };
    auto note_overflow = [&](int parity) {
        bool over = false;
#pragma unroll
        for (int g = 0; g < XG; ++g) over |= !(run_s[g] < 1.0e30f);  // or NaN
        if (__any(over) && lane == 0) over_flag[parity] = 1;
    };
    // One attempt at the streamed range: prologue loads, the ring of steps, the short last tile.  Returns whether the
    // block has to start over (FDH, fast form only; the value is the same in every wavefront of the block).
    auto run_attempt = [&](auto form) -> bool {
        constexpr bool EXACT = decltype(form)::exact;
        constexpr bool WATCH = (MODE == MODE_FDH) && !EXACT;  // the fast form watches for sums that leave the float range
        int overflow = 0;  // wave-uniform
        auto step = [&](int64_t t, const uint16_t *cur, uint16_t *nxt) {
            if (t + PF < t_end) {
                int32_t rows[NR];
                rows_from_lds(t + PF, cur, rows);
                issue_group(t + PF, rows, nxt);
            }
            if (MODE == MODE_FDH && EXACT) raise_reference(cur, BY);
            // The flag that the previous step may have raised (every wavefront of the block reads it between the same
            // two barriers, so all of them see the same value); the read lands under the work on this tile.
            int seen = 0;
            if (WATCH && t != t_begin) seen = over_flag[(int)((t - t_begin - 1) & 1)];
            // d = 256: few tiles per block and a kernel at the edge of its register budget; measured slower there
            if (MODE == MODE_FWD && D <= 128 && t != t_begin) {  // the first tile has no maximum to lean on
                float m0[XG], s0[XG];
                bool over = false;
#pragma unroll
                for (int g = 0; g < XG; ++g) {
                    m0[g] = run_m[g];
                    s0[g] = run_s[g];
                }
                process_tile(t, cur, Full{}, Lazy{});
#pragma unroll
                for (int g = 0; g < XG; ++g) over |= !(run_s[g] < 1.0e30f);  // near overflow (or NaN): the merges of
                                                                                  // half-waves and of split runs add up to 16 such sums
                if (__any(over)) {
#pragma unroll
                    for (int g = 0; g < XG; ++g) {
                        run_m[g] = m0[g];
                        run_s[g] = s0[g];
                    }
                    process_tile(t, cur, Full{}, Exact{});
                }
            } else {
                process_tile(t, cur, Full{}, Exact{});
            }
            pin_results();
            if (WATCH) {
                note_overflow((int)((t - t_begin) & 1));
                overflow |= __builtin_amdgcn_readfirstlane(seen);
            }
            wait_for_next(t);
            barrier_keep_loads();
        };
        if (WATCH && tid < 2) over_flag[tid] = 0;  // visible behind the barrier that follows the first loads
        if (t_begin < t_end) {
            int32_t rows[PF][NR];
#pragma unroll
            for (int j = 0; j < PF; ++j)
                if (t_begin + j < t_end) rows_from_global(t_begin + j, rows[j]);
#pragma unroll
            for (int j = 0; j < PF; ++j)
                if (t_begin + j < t_end) issue_group(t_begin + j, rows[j], buf_at(j));
        }
        wait_for_next(t_begin - 1);
        barrier_keep_loads();
        if (WATCH && t_begin < t_end) {  // reference of the fast form: the largest score among the first 32 candidates
            const int64_t left = n_y - t_begin * BY;
            float tmax[XG];
            tile_max(buf_at(0), 1, left < BY ? (int)left : BY, tmax);
#pragma unroll
            for (int g = 0; g < XG; ++g) run_m[g] = tmax[g];
        }
        if (NBUF == 4) {
            for (int64_t t = t_begin; t < t_stop; t += 4) {
                step(t, buf0, buf3);
                if (t + 1 >= t_stop || overflow) break;
                step(t + 1, buf1, buf0);
                if (t + 2 >= t_stop || overflow) break;
                step(t + 2, buf2, buf1);
                if (t + 3 >= t_stop || overflow) break;
                step(t + 3, buf3, buf2);
                if (overflow) break;
            }
        } else if (NBUF == 3) {
            for (int64_t t = t_begin; t < t_stop; t += 3) {
                step(t, buf0, buf2);
                if (t + 1 >= t_stop || overflow) break;
                step(t + 1, buf1, buf0);
                if (t + 2 >= t_stop || overflow) break;
                step(t + 2, buf2, buf1);
                if (overflow) break;
            }
        } else if (NBUF == 2) {
            for (int64_t t = t_begin; t < t_stop; t += 2) {
                step(t, buf0, buf1);
                if (t + 1 >= t_stop || overflow) break;
                step(t + 1, buf1, buf0);
                if (overflow) break;
            }
        } else {
            for (int64_t t = t_begin; t < t_stop && !overflow; ++t) {
                const int s = (int)((t - t_begin) & 1);
                step(t, buf_at(s), buf_at(s ^ 1));
            }
        }
        if (tail_ragged && !overflow) {  // its group was issued with the others, and the last wait above was for all loads
            const uint16_t *last = buf_at((int)((t_stop - t_begin) % NB));
            if (MODE == MODE_FDH && EXACT) raise_reference(last, (int)(n_y - t_stop * BY));
            process_tile(t_stop, last, Ragged{}, Exact{});
            if (WATCH) note_overflow(0);
            __syncthreads();  // the dE epilogue reuses the tile buffers
        }
        if (WATCH) {
            // the flags of the last step and of the short tile have not been read yet (the last barrier is behind us)
            if (!overflow) overflow = __builtin_amdgcn_readfirstlane(over_flag[0] | over_flag[1]);
            if (overflow) {  // loads of later tiles may still be in flight into the ring: let them land
                wait_vm<0>();
                __syncthreads();
            }
        }
        return overflow != 0;
    };
    if (run_attempt(FastTag{})) {
        if constexpr (MODE == MODE_FDH) {  // start over in the exact form
#pragma unroll
            for (int g = 0; g < XG; ++g) {
                run_m[g] = -INFINITY;
                run_s[g] = 0.f;
#pragma unroll
                for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[g][mb][q] = 0.f;
            }
            run_attempt(ExactTag{});
        }
    }


    // =====================================================================================================  epilogues
    if (MODE == MODE_FWD) {
#pragma unroll
        for (int g = 0; g < XG; ++g) {
            // merge the two halves of the candidates that lanes (lo,0) and (lo,1) hold for the same position
            float rm = run_m[g], rs = run_s[g];
            {
                const float m2 = __shfl_xor(rm, 32, 64), s2 = __shfl_xor(rs, 32, 64);
                const float M = fmaxf(rm, m2);
                if (M > -INFINITY) {
                    rs = rs * __builtin_amdgcn_exp2f(rm - M) + s2 * __builtin_amdgcn_exp2f(m2 - M);
                    rm = M;
                }
            }
            const int64_t x = xb * XPB + (xgrp * XG + g) * 32 + lo;
            if (a.splits > 1) {
                if (x_ok[g] && hi == 0) {
                    a.part_m[(int64_t)split * a.N + x] = rm;
                    a.part_s[(int64_t)split * a.N + x] = rs;
                }
                continue;
            }
            float op = 0.f;
            if (x_ok[g]) op = half_row_dot<D>(xr[g], a.E + (int64_t)a.tgt[xrow[g]] * D, hi);
            op += __shfl_xor(op, 32, 64);
            if (x_ok[g] && hi == 0) {
                const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[xrow[g]] : 1.f);
                const float o2 = op * kLog2e;
                const float M = (w != 0.f) ? fmaxf(rm, o2) : rm;
                const float tot = rs * __builtin_amdgcn_exp2f(rm - M) + w * __builtin_amdgcn_exp2f(o2 - M);
                const float l = (M + __builtin_amdgcn_logf(tot)) * kLn2;
                a.lse[xrow[g]] = l;
                a.loss[xrow[g]] = l - op;
                // what a backward call that reuses this call's preparation needs per position, short of the upstream
                // gradient: the correct item's coefficient w p+ - 1 and the exponent offset of the dE pass
                const float nl = -l * kLog2e;
                a.coef[xrow[g]] = w * __builtin_amdgcn_exp2f(fmaf(op, kLog2e, nl)) - 1.f;
                a.de_const[x] = __float_as_uint(nl);
            }
        }
    } else if (MODE == MODE_FDH) {
#pragma unroll
        for (int g = 0; g < XG; ++g) {
            const int64_t x = xb * XPB + (xgrp * XG + g) * 32 + lo;
            const float rm = run_m[g];
            const float rs = run_s[g] + __shfl_xor(run_s[g], 32, 64);  // the two halves share the reference
            if (splits > 1) {  // partial (reference, sum, rows) of this part of the candidate range; the merge finishes
                if (x_ok[g]) {
                    const int64_t slot = (int64_t)split * part_rows + (x - part_x0);
                    if (hi == 0 && half == 0) {
                        a.part_m[slot] = rm;
                        a.part_s[slot] = rs;
                    }
                    float *dst = a.part_dH + slot * D;
#pragma unroll
                    for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq)
                            *reinterpret_cast<float4 *>(dst + (half * MBH + mb) * 32 + qq * 8 + hi * 4) = make_float4(
                                acc[g][mb][qq * 4], acc[g][mb][qq * 4 + 1], acc[g][mb][qq * 4 + 2], acc[g][mb][qq * 4 + 3]);
                }
                continue;
            }
            float op = 0.f;
            const uint16_t *erow = a.E + (x_ok[g] ? (int64_t)a.tgt[xrow[g]] : 0) * D;
            if (x_ok[g]) op = half_row_dot<D>(xr[g], erow, hi);
            op += __shfl_xor(op, 32, 64);
            if (x_ok[g]) {
                const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[xrow[g]] : 1.f);
                const float o2 = op * kLog2e;
                const float M = (w != 0.f) ? fmaxf(rm, o2) : rm;
                const float e1 = __builtin_amdgcn_exp2f(rm - M), e2 = (w != 0.f) ? w * __builtin_amdgcn_exp2f(o2 - M) : 0.f;
                const float tot = rs * e1 + e2;
                const float l = (M + __builtin_amdgcn_logf(tot)) * kLn2;
                const float inv = e1 / tot;        // 2^(reference) / sum of all live exponentials
                const float cpos = e2 / tot - 1.f;  // coefficient of the correct item, w p+ - 1
                if (hi == 0 && half == 0) {
                    a.lse[xrow[g]] = l;
                    a.loss[xrow[g]] = l - op;
                    a.coef[xrow[g]] = cpos;
                    a.de_const[x] = __float_as_uint(-l * kLog2e);
                }
#pragma unroll
                for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const int col = (half * MBH + mb) * 32 + qq * 8 + hi * 4;
                        const uint2 ev = *reinterpret_cast<const uint2 *>(erow + col);
                        *reinterpret_cast<float4 *>(a.U + xrow[g] * D + col) =
                            make_float4(fmaf(cpos, bf16_lo(ev.x), acc[g][mb][qq * 4 + 0] * inv), fmaf(cpos, bf16_hi(ev.x), acc[g][mb][qq * 4 + 1] * inv),
                                        fmaf(cpos, bf16_lo(ev.y), acc[g][mb][qq * 4 + 2] * inv), fmaf(cpos, bf16_hi(ev.y), acc[g][mb][qq * 4 + 3] * inv));
                    }
            }
        }
    } else if (MODE == MODE_DH) {
#pragma unroll
        for (int g = 0; g < XG; ++g) {
            const int64_t x = xb * XPB + (xgrp * XG + g) * 32 + lo;
            if (splits > 1) {
                if (x_ok[g]) {
                    float *dst = a.part_dH + ((int64_t)split * part_rows + (x - part_x0)) * D;
#pragma unroll
                    for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq)
                            *reinterpret_cast<float4 *>(dst + (half * MBH + mb) * 32 + qq * 8 + hi * 4) = make_float4(
                                acc[g][mb][qq * 4], acc[g][mb][qq * 4 + 1], acc[g][mb][qq * 4 + 2], acc[g][mb][qq * 4 + 3]);
                }
                continue;
            }
            float op = 0.f;
            const uint16_t *erow = a.E + (x_ok[g] ? (int64_t)a.tgt[xrow[g]] : 0) * D;
            if (x_ok[g]) op = half_row_dot<D>(xr[g], erow, hi);
            op += __shfl_xor(op, 32, 64);
            if (x_ok[g]) {
                const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[xrow[g]] : 1.f);
                const float pp = __builtin_amdgcn_exp2f(fmaf(op, kLog2e, cx[g]));
                const float cpos = w * pp - 1.f;  // coefficient of the correct item before the upstream gradient
                const float gg = a.g ? a.g[xrow[g]] : 1.f;
                if (a.write_consts && hi == 0 && half == 0) a.coef[xrow[g]] = gg * cpos;
#pragma unroll
                for (int mb = 0; mb < MBH; ++mb)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const int col = (half * MBH + mb) * 32 + qq * 8 + hi * 4;
                        const uint2 ev = *reinterpret_cast<const uint2 *>(erow + col);
                        const float v0 = gg * fmaf(cpos, bf16_lo(ev.x), acc[g][mb][qq * 4 + 0]);
                        const float v1 = gg * fmaf(cpos, bf16_hi(ev.x), acc[g][mb][qq * 4 + 1]);
                        const float v2 = gg * fmaf(cpos, bf16_lo(ev.y), acc[g][mb][qq * 4 + 2]);
                        const float v3 = gg * fmaf(cpos, bf16_hi(ev.y), acc[g][mb][qq * 4 + 3]);
                        if (a.dH_bf16) {
                            *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.dH) + xrow[g] * D + col) =
                                make_uint2(pack2(v0, v1), pack2(v2, v3));
                        } else {
                            *reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + xrow[g] * D + col) =
                                make_float4(v0, v1, v2, v3);
                        }
                    }
            }
        }
    } else {
        // dE_neg^T sits in the accumulators with the hidden index in registers and the candidate row on the lanes.
        // Turn each 32x32 block round through LDS (the streamed tiles are dead by now) so that one atomic
        // instruction adds 32 consecutive floats to each of two table rows.
        float *tbuf = EPI_IN_TILES ? reinterpret_cast<float *>(buf_at(wave & 1)) + (wave >> 1) * (32 * 33)  // 2 per buffer
                                   : epi_own + wave * (32 * 33);
        int64_t *xrow_s = EPI_IN_TILES ? reinterpret_cast<int64_t *>(reinterpret_cast<float *>(buf0) + 2 * (32 * 33))
                                       : reinterpret_cast<int64_t *>(epi_own + NW * (32 * 33));
#pragma unroll
        for (int g = 0; g < XG; ++g) xrow_s[(xgrp * XG + g) * 32 + lo] = x_ok[g] ? xrow[g] : -1;  // both half-waves agree
        __syncthreads();
#pragma unroll
        for (int g = 0; g < XG; ++g) {
#pragma unroll
            for (int mb = 0; mb < MBH; ++mb) {
#pragma unroll
                for (int q = 0; q < 16; ++q) tbuf[lo * 33 + (q / 4) * 8 + hi * 4 + (q % 4)] = acc[g][mb][q];
                __syncthreads();
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int xl = r * 2 + hi;
                    const int64_t row = xrow_s[(xgrp * XG + g) * 32 + xl];
                    const float v = tbuf[xl * 33 + lo];
                    if (row >= 0) unsafeAtomicAdd(a.dE + row * D + (half * MBH + mb) * 32 + lo, v);
                }
                __syncthreads();
            }
        }
    }
}

template <int D, int MODE, int BY, int NW, int XG, int MINB, int NBUF, int DS, bool FILTER>
__global__ __launch_bounds__(NW * 64, MINB) void tile_kernel(TileArgs a)
{
    typedef TileGeom<D, MODE, BY, NW, XG, NBUF, DS> G;
    __shared__ __attribute__((aligned(1024))) uint16_t buf0[G::BUF0];
    __shared__ __attribute__((aligned(1024))) uint16_t buf1[G::BUF1];
    __shared__ __attribute__((aligned(1024))) uint16_t buf2[G::BUF2];
    __shared__ __attribute__((aligned(1024))) uint16_t buf3[G::BUF3];
    __shared__ __attribute__((aligned(16))) float epi_own[G::EPI_OWN];
    tile_body<D, MODE, BY, NW, XG, NBUF, DS, FILTER>(a, (int64_t)blockIdx.x, buf0, buf1, buf2, buf3, epi_own);
}

// The dH and the dE pass of one backward call in a single launch: with few positions neither pass fills the chip on
// its own (c2: 320 + 256 blocks of one wavefront per SIMD each), and both are bound by latencies rather than by any
// unit, so they overlap almost completely.  The dE blocks (correct-item scatter first) lead the grid, being the longer
// ones.  Both roles share the LDS arrays; neither reads what the other writes (coef and de_const come from the
// forward call, or from bwd_pre_kernel when its preparation is not reused).
template <int D, int BY, int XG_DH, int XG_DE, int NBUF, bool FILTER>
__global__ __launch_bounds__(256, 2) void tile_bwd_kernel(TileArgs a_dh, TileArgs a_de, int64_t de_blocks)
{
    typedef TileGeom<D, MODE_DH, BY, 4, XG_DH, NBUF, 1> GH;
    typedef TileGeom<D, MODE_DE, BY, 4, XG_DE, NBUF, 1> GE;
    constexpr int B0 = GH::BUF0 > GE::BUF0 ? GH::BUF0 : GE::BUF0, B1 = GH::BUF1 > GE::BUF1 ? GH::BUF1 : GE::BUF1;
    constexpr int B2 = GH::BUF2 > GE::BUF2 ? GH::BUF2 : GE::BUF2, B3 = GH::BUF3 > GE::BUF3 ? GH::BUF3 : GE::BUF3;
    __shared__ __attribute__((aligned(1024))) uint16_t buf0[B0];
    __shared__ __attribute__((aligned(1024))) uint16_t buf1[B1];
    __shared__ __attribute__((aligned(1024))) uint16_t buf2[B2];
    __shared__ __attribute__((aligned(1024))) uint16_t buf3[B3];
    __shared__ __attribute__((aligned(16))) float epi_own[GE::EPI_OWN];
    // grid order: the dE role (correct-item scatter, then its tiles) ahead of the dH role (zeroing of padded rows, then
    // its tiles); measured faster on c2 than tiles first
    const int64_t b = (int64_t)blockIdx.x;
    if (b < de_blocks)
        tile_body<D, MODE_DE, BY, 4, XG_DE, NBUF, 1, FILTER>(a_de, b, buf0, buf1, buf2, buf3, epi_own);
    else
        tile_body<D, MODE_DH, BY, 4, XG_DH, NBUF, 1, FILTER>(a_dh, b - de_blocks, buf0, buf1, buf2, buf3, epi_own);
}

// Per valid position, ahead of a fused backward launch that does not reuse the forward call's constants: the coefficient of the correct item g (w p+ - 1) for the
// scatter, and the exponent offset -lse log2e and g of the dE coefficients g exp(o - lse) = g 2^(o log2e - lse log2e)
// under the compacted index.  D/8 lanes per position share the scalar product with the correct item's row.
template <int D>
__global__ __launch_bounds__(256) void bwd_pre_kernel(TileArgs a)
{
    constexpr int LPR = D / 8;
    constexpr int PPB = 256 / LPR;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t x = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
    const int c = threadIdx.x % LPR;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float op = 0.f;
    if (ok) {
        float h[8], e[8];
        load8(a.H + row * D + c * 8, h);
        load8(a.E + (int64_t)a.tgt[row] * D + c * 8, e);
#pragma unroll
        for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) op += __shfl_xor(op, off, 64);
    if (ok && c == 0) {
        const float nl = -a.lse_in[row] * kLog2e;
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float gg = a.g ? a.g[row] : 1.f;
        a.coef[row] = gg * (w * __builtin_amdgcn_exp2f(fmaf(op, kLog2e, nl)) - 1.f);
        a.de_const[x] = __float_as_uint(nl);
        a.de_const[a.N + x] = __float_as_uint(gg);
    }
}

// ---------------------------------------------------------------------------------------------------------------------
// Merges of split runs (few positions, many candidates: the candidate range is split over blocks).
template <int D>
__global__ __launch_bounds__(256) void fwd_merge_kernel(TileArgs a)
{
    // 8 lanes per position: each takes the chunks c, c+8, ... of the row for the correct-item score
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t x = ((int64_t)blockIdx.x * 256 + threadIdx.x) / 8;
    const int c = threadIdx.x & 7;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float op = 0.f;
    if (ok) {
        const uint16_t *hp = a.H + row * D, *ep = a.E + (int64_t)a.tgt[row] * D;
        for (int ch = c; ch < D / 8; ch += 8) {
            float h[8], e[8];
            load8(hp + ch * 8, h);
            load8(ep + ch * 8, e);
#pragma unroll
            for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
        }
    }
    op += __shfl_xor(op, 1, 64);
    op += __shfl_xor(op, 2, 64);
    op += __shfl_xor(op, 4, 64);
    if (ok && c == 0) {
        float m = -INFINITY, s = 0.f;
        for (int sp = 0; sp < a.splits; ++sp) {
            const float m2 = a.part_m[(int64_t)sp * a.N + x], s2 = a.part_s[(int64_t)sp * a.N + x];
            const float M = fmaxf(m, m2);
            if (M > -INFINITY) {
                s = s * __builtin_amdgcn_exp2f(m - M) + s2 * __builtin_amdgcn_exp2f(m2 - M);
                m = M;
            }
        }
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float o2 = op * kLog2e;
        const float M = (w != 0.f) ? fmaxf(m, o2) : m;
        const float tot = s * __builtin_amdgcn_exp2f(m - M) + w * __builtin_amdgcn_exp2f(o2 - M);
        const float l = (M + __builtin_amdgcn_logf(tot)) * kLn2;
        a.lse[row] = l;
        a.loss[row] = l - op;
        const float nl = -l * kLog2e;  // as in the unsplit epilogue
        a.coef[row] = w * __builtin_amdgcn_exp2f(fmaf(op, kLog2e, nl)) - 1.f;
        a.de_const[x] = __float_as_uint(nl);
    }
}

// TAIL_XPB > 0: the merge of the last-round split of the dH pass (position blocks of TAIL_XPB rows), same plan as there.
template <int D, int TAIL_XPB = 0>
__global__ __launch_bounds__(256) void dh_merge_kernel(TileArgs a)
{
    constexpr int LPR = D / 8;  // lanes per position, 8 columns each
    static_assert(64 % LPR == 0 || LPR % 64 == 0, "row must tile the wavefront");
    constexpr int PPB = 256 / LPR;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    int64_t x = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
    int64_t part_rows = a.N, part_x0 = 0;
    int splits = a.splits;
    if (TAIL_XPB > 0) {
        const TailPlan tp = tail_plan((n_pos + TAIL_XPB - 1) / TAIL_XPB, a.tail_slots);
        part_rows = tp.tail * TAIL_XPB;
        part_x0 = tp.whole * TAIL_XPB;
        splits = tp.splits;
        if (x >= part_rows) x = n_pos;  // nothing to merge here
        else x += part_x0;
    }
    const int c = threadIdx.x % LPR;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float h[8], e[8], sum[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) h[t] = e[t] = sum[t] = 0.f;
    float op = 0.f;
    if (ok) {
        load8(a.H + row * D + c * 8, h);
        load8(a.E + (int64_t)a.tgt[row] * D + c * 8, e);
#pragma unroll
        for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
        for (int sp = 0; sp < splits; ++sp) {
            float v[8];
            load8(a.part_dH + ((int64_t)sp * part_rows + (x - part_x0)) * D + c * 8, v);
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] += v[t];
        }
    }
    // rows never straddle a wavefront when LPR <= 64; for D = 512 this kernel is not instantiated
#pragma unroll
    for (int off = 1; off < LPR && off < 64; off <<= 1) op += __shfl_xor(op, off, 64);
    if (ok) {
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float pp = __builtin_amdgcn_exp2f((op - a.lse_in[row]) * kLog2e);
        const float cpos = w * pp - 1.f;
        const float g = a.g ? a.g[row] : 1.f;
        if (c == 0 && a.write_consts) a.coef[row] = g * cpos;  // for a scatter in a later launch; the fused launch has its own
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = g * fmaf(cpos, e[t], sum[t]);
        if (a.dH_bf16) {
            *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.dH) + row * D + c * 8) =
                make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
        } else {
            float4 *out = reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + row * D + c * 8);
            out[0] = make_float4(v[0], v[1], v[2], v[3]);
            out[1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
}

// Merge of a split FDH pass: the parts of a position's candidate range come with their own reference m_s, sum l_s and
// unnormalised rows A_s; with M = max m_s the position's sum is sum_s l_s 2^(m_s - M) and its rows sum_s A_s 2^(m_s - M).
// Then as in the unsplit epilogue: the correct item's term, lse, loss, the constants of the backward pass, and U.
template <int D, int TAIL_XPB = 0>
__global__ __launch_bounds__(256) void fdh_merge_kernel(TileArgs a)
{
    constexpr int LPR = D / 8;  // lanes per position, 8 columns each
    static_assert(64 % LPR == 0, "a row must not straddle wavefronts");
    constexpr int PPB = 256 / LPR;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    int64_t x = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
    int64_t part_rows = a.N, part_x0 = 0;
    int splits = a.splits;
    if constexpr (TAIL_XPB > 0) {
        const TailPlan tp = tail_plan((n_pos + TAIL_XPB - 1) / TAIL_XPB, a.tail_slots);
        part_rows = tp.tail * TAIL_XPB;
        part_x0 = tp.whole * TAIL_XPB;
        splits = tp.splits;
        if (x >= part_rows) x = n_pos;  // nothing to merge here
        else x += part_x0;
    }
    const int c = threadIdx.x % LPR;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float h[8], e[8], sum[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) h[t] = e[t] = sum[t] = 0.f;
    float op = 0.f, M = -INFINITY, l = 0.f;
    if (ok) {
        load8(a.H + row * D + c * 8, h);
        load8(a.E + (int64_t)a.tgt[row] * D + c * 8, e);
#pragma unroll
        for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
        for (int sp = 0; sp < splits; ++sp) M = fmaxf(M, a.part_m[(int64_t)sp * part_rows + (x - part_x0)]);
        for (int sp = 0; sp < splits; ++sp) {
            const int64_t slot = (int64_t)sp * part_rows + (x - part_x0);
            const float ms = a.part_m[slot];
            if (ms == -INFINITY) continue;  // a part without candidates
            const float sc = __builtin_amdgcn_exp2f(ms - M);
            l = fmaf(a.part_s[slot], sc, l);
            float v[8];
            load8(a.part_dH + slot * D + c * 8, v);
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] = fmaf(v[t], sc, sum[t]);
        }
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) op += __shfl_xor(op, off, 64);
    if (ok) {
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float o2 = op * kLog2e;
        const float Mx = (w != 0.f) ? fmaxf(M, o2) : M;
        const float e1 = __builtin_amdgcn_exp2f(M - Mx), e2 = (w != 0.f) ? w * __builtin_amdgcn_exp2f(o2 - Mx) : 0.f;
        const float tot = l * e1 + e2;
        const float lse = (Mx + __builtin_amdgcn_logf(tot)) * kLn2;
        const float inv = e1 / tot, cpos = e2 / tot - 1.f;
        if (c == 0) {
            a.lse[row] = lse;
            a.loss[row] = lse - op;
            a.coef[row] = cpos;
            a.de_const[x] = __float_as_uint(-lse * kLog2e);
        }
        float4 *out = reinterpret_cast<float4 *>(a.U + row * D + c * 8);
        out[0] = make_float4(fmaf(cpos, e[0], sum[0] * inv), fmaf(cpos, e[1], sum[1] * inv), fmaf(cpos, e[2], sum[2] * inv), fmaf(cpos, e[3], sum[3] * inv));
        out[1] = make_float4(fmaf(cpos, e[4], sum[4] * inv), fmaf(cpos, e[5], sum[5] * inv), fmaf(cpos, e[6], sum[6] * inv), fmaf(cpos, e[7], sum[7] * inv));
    }
}

template <int D, bool FILE_G>
__global__ __launch_bounds__(256) void dh_scale_kernel(TileArgs a)
{
    const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (FILE_G) {
        const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
        if (chunk < n_pos) a.de_const[a.N + chunk] = __float_as_uint(a.g ? a.g[pos_row(a, chunk)] : 1.f);
    }
    dh_scale_chunk<D>(a, chunk);
}

// ---------------------------------------------------------------------------------------------------------------------
// Blocks of one kernel instantiation that the current device holds at once.  The answer is cached per instantiation
// (the template makes the static array one per kernel) and per device ordinal.
constexpr int kMaxDevices = 64;
template <typename K>
int resident_blocks(K kernel, int threads)
{
    static std::atomic<int> cache[kMaxDevices];  // 0 = not asked yet
    int per_cu = 0, dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (cached) {
        const int v = cache[dev].load(std::memory_order_relaxed);
        if (v > 0) return v;
    }
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1 ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1)
        return 256;
    if (cached) cache[dev].store(per_cu * cus, std::memory_order_relaxed);
    return per_cu * cus;
}

// Split factor in [1, max_splits] that wastes the least of the last round of blocks; ties go to the smaller factor,
// and a factor is only raised for a gain of at least five percent.
inline int pick_splits(int64_t xblocks, int max_splits, int slots, bool cheap_merge, bool atomic_merge)
{
    // enough blocks already: a split costs partial results and a merge.  Where the merge is cheap (forward: two floats
    // per position and split) a grid of a few rounds is still split to even out its last round.  The dE pass merges by
    // atomics under the other blocks' matrix work: a grid of less than two rounds is split when that fills the last
    // round at least 15 % better (c4: 391 blocks on 512 slots, 405 us unsplit, 367 us in 5 splits).
    double min_gain = 1.05;
    if (xblocks * 4 > slots && !(cheap_merge && xblocks > slots && xblocks < 8 * (int64_t)slots)) {
        if (!(atomic_merge && xblocks < 2 * (int64_t)slots)) return 1;
        min_gain = 1.15;
    }
    int best = 1;
    double best_eff = 0.0;
    for (int s = 1; s <= max_splits; ++s) {
        const int64_t blocks = xblocks * s;
        const int64_t rounds = (blocks + slots - 1) / slots;
        const double eff = (double)blocks / (double)(rounds * slots);
        // forward pass: the block count is an upper bound when positions are padded, and every split repeats the
        // block prologue: the first factor that fills the last round reasonably is taken (c5: 2 instead of 4, 394 -> 361 us)
        if (cheap_merge && eff >= 0.88) return s;
        if (eff > best_eff * (s == 1 ? 0.0 : min_gain)) {
            best_eff = eff;
            best = s;
        }
    }
    return best;
}

// Split factor and leading blocks of one pass; returns the number of blocks of its grid (0: nothing to do).
// fine: the pass shares its launch with another role that fills most block slots; if it splits at all, it splits as
// finely as allowed, so that its blocks fill the gaps (c4: the fused backward launch 704 -> 671 us with 16 instead of 10).
template <int MODE>
int64_t plan_tile_grid(TileArgs &a, int64_t n_x, int xpb, int threads, int slots, bool fine = false)
{
    const int64_t xblocks = (n_x + xpb - 1) / xpb;
    if (xblocks == 0) return 0;
    if (MODE == MODE_DE) {
        // every split of the position range pays n_cols * d atomics: keep them below about a quarter of the matrix
        // time of the pass (4 n_cols d N flop at ~1 PFLOP/s against ~300 G atomics/s) => splits <= 3e-4 N
        const int cap = (int)(a.N * 5e-4) < 8 ? 8 : (int)(a.N * 5e-4);
        if (a.splits > cap) a.splits = cap;
    }
    const int max_splits = a.splits;
    a.splits = pick_splits(xblocks, a.splits, slots, MODE == MODE_FWD, MODE == MODE_DE);
    if (fine && a.splits > 1) a.splits = max_splits;
    int64_t blocks = xblocks * a.splits;
    if (MODE == MODE_DE) {  // the latency-bound scatter blocks go first so that they run under the matrix work
        a.pos_blocks = a.scatter_apart ? 0 : (a.N + kPosChunk - 1) / kPosChunk;
        blocks += a.pos_blocks;
    }
    if (MODE == MODE_DH) {
        a.pad_blocks = (a.pos_mask || a.validate) ? (a.N + threads - 1) / threads : 0;
        blocks += a.pad_blocks;
    }
    if (MODE == MODE_DE && a.scale_blocks > 0) {  // wanted by the caller: dH = grad_loss * U in trailing blocks
        a.scale_block0 = blocks;
        a.scale_blocks = (a.N * (a.d / 8) + (int64_t)threads * kScaleChunks - 1) / ((int64_t)threads * kScaleChunks);
        blocks += a.scale_blocks;
    }
    return blocks;
}

template <int D, int MODE, int BY, int NW, int XG, int MINB, int NBUF, int DS = 1, bool FILTER = false>
hipError_t launch_tile_kernel(TileArgs &a, int64_t n_x, hipStream_t stream)
{
    const int slots = resident_blocks(tile_kernel<D, MODE, BY, NW, XG, MINB, NBUF, DS, FILTER>, NW * 64);
    constexpr int XPB = (NW / DS) * XG * 32;
    int64_t blocks = plan_tile_grid<MODE>(a, n_x, XPB, NW * 64, slots);
    if (blocks == 0) return hipSuccess;
    a.tail_slots = 0;
    if ((MODE == MODE_DH || MODE == MODE_FDH) && D > 128 && a.splits == 1 && n_x > kTailRows && (int64_t)slots * XPB <= kTailRows) {
        a.tail_slots = slots;  // last-round split: at most `slots` blocks more than position blocks
        blocks += slots;
    }
    ProfScope prof(MODE == MODE_FWD ? PROF_TILE_FWD : (MODE == MODE_DH ? PROF_TILE_DH : (MODE == MODE_DE ? PROF_TILE_DE : PROF_TILE_FDH)), stream);
    hipLaunchKernelGGL((tile_kernel<D, MODE, BY, NW, XG, MINB, NBUF, DS, FILTER>), dim3((unsigned)blocks), dim3(NW * 64), 0, stream, a);
    return hipGetLastError();
}

template <int D, int XG_DH, int XG_DE, bool FILTER = false>
hipError_t launch_bwd_kernel(TileArgs &a_dh, TileArgs &a_de, hipStream_t stream)
{
    constexpr int BY = 8192 / D, NBUF = 4;
    const int slots = resident_blocks(tile_bwd_kernel<D, BY, XG_DH, XG_DE, NBUF, FILTER>, 256);
    const int64_t de_blocks = plan_tile_grid<MODE_DE>(a_de, a_de.n_cols, 4 * XG_DE * 32, 256, slots);
    const int64_t dh_blocks = plan_tile_grid<MODE_DH>(a_dh, a_dh.N, 4 * XG_DH * 32, 256, slots, true);
    if (de_blocks + dh_blocks == 0) return hipSuccess;
    ProfScope prof(PROF_TILE_BWD, stream);
    hipLaunchKernelGGL((tile_bwd_kernel<D, BY, XG_DH, XG_DE, NBUF, FILTER>), dim3((unsigned)(de_blocks + dh_blocks)), dim3(256), 0, stream,
                       a_dh, a_de, de_blocks);
    return hipGetLastError();
}

template <int D>
hipError_t launch_for_d(int pass, TileArgs a, hipStream_t stream)
{
    // Forward: 16 KiB of bf16 per tile buffer (128 rows at d = 64, 32 rows at d = 256); three blocks per compute unit
    // at d = 64 (register budget 168), else two.
    constexpr int BY = 8192 / D;
    // d = 256, forward: tiles of four sub-tiles, so that the software-pipelined loop (score product of sub-tile k + 1
    // under the softmax arithmetic of sub-tile k) has something to overlap in three phases out of four.
    constexpr int BY_F = (D <= 128) ? BY : 128;
    constexpr int MINB_F = (D <= 64) ? 3 : 2;
    // d = 256: every block streams the whole other operand from L2 (about 12 TB/s over the chip for direct-to-LDS
    // loads), so the rows it keeps stationary decide the traffic: eight wavefronts per block, one block per compute
    // unit.  The backward accumulators for all columns (d/2 registers) plus the stationary rows (d/4) leave little of
    // the 256-register budget: operands are read two at a time there.
    constexpr int NW_L = (D <= 128) ? 4 : 8;
    constexpr int DS_B = 1;
    constexpr int BY_B = BY;  // d = 256: tiles of 64 rows measured 3-6 % slower
    constexpr int MINB = (D <= 128) ? 2 : 1;   // backward: 256 registers per wavefront
    // LDS buffers in flight, 18 KiB each: three blocks per compute unit leave room for three of them, two blocks or
    // one for four.  d = 256: two 66-KiB buffers in the forward pass; three buffers in the backward passes (measured:
    // dE 5 % faster than with two, dH unchanged, four no better).
    constexpr int NBUF_F = (D <= 64) ? 3 : (D <= 128 ? 4 : 2);
    constexpr int NBUF_B = (D <= 128) ? 4 : 3;
    constexpr int NBUF_FDH = 4;  // d = 256: 2 % faster than three (the dE pass: 20 % slower)
    // Two groups of stationary rows per wavefront use each LDS operand for two matrix instructions; the backward
    // accumulators leave room for that up to d = 64.
    constexpr int XG_F = 2;
    constexpr int XG_B = (D <= 64) ? 2 : 1;
    hipError_t e = hipSuccess;
    // Two groups want 256 stationary rows per block: worth it when that still gives about two blocks per compute
    // unit, either directly or because the streamed range is being split anyway.
    auto wide = [&](int64_t n_x, bool may_split) {
        const int64_t xb = (n_x + NW_L * 64 - 1) / (NW_L * 64);
        if (NW_L == 8) return xb >= 256;  // one block per compute unit: at least one full round of the coarser unit
        return xb >= 300 || (may_split && xb < 120 && xb * a.splits >= 480);
    };
    switch (pass) {
    case TILE_PASS_FWD:
        if constexpr (D > 128) {  // one group of stationary rows per wavefront: registers for two score tiles in flight
            e = launch_tile_kernel<D, MODE_FWD, BY_F, NW_L, 1, 1, NBUF_F>(a, a.N, stream);
        } else if (wide(a.N, true))
            e = launch_tile_kernel<D, MODE_FWD, BY, NW_L, XG_F, 2, 4>(a, a.N, stream);
        else
            e = launch_tile_kernel<D, MODE_FWD, BY, NW_L, 1, MINB_F, NBUF_F>(a, a.N, stream);
        if (e == hipSuccess && a.splits > 1) {
            ProfScope prof(PROF_FWD_MERGE, stream);
            hipLaunchKernelGGL((fwd_merge_kernel<D>), dim3((unsigned)((a.N * 8 + 255) / 256)), dim3(256), 0, stream, a);
            e = hipGetLastError();
        }
        return e;
    case TILE_PASS_DH: {
        bool done = false;
        if constexpr (XG_B == 2) {
            if (wide(a.N, true)) {
                e = launch_tile_kernel<D, MODE_DH, BY_B, 4, 2, MINB, NBUF_B>(a, a.N, stream);
                done = true;
            }
        }
        if (!done && a.filter_log2 > -INFINITY) {
            if constexpr (D > 128) e = launch_tile_kernel<D, MODE_DH, BY_B, NW_L, 1, MINB, NBUF_B, DS_B, true>(a, a.N, stream);
            else e = hipErrorInvalidValue;  // smaller hidden sizes filter in the fused launch
        } else if (!done) e = launch_tile_kernel<D, MODE_DH, BY_B, NW_L, 1, MINB, NBUF_B, DS_B>(a, a.N, stream);
        if constexpr (D > 128) {
            if (e == hipSuccess && a.tail_slots > 0) {  // rows of the split last round: at most half the chip's blocks
                constexpr int PPB = 256 / (D / 8), XPB_L = NW_L * 32;
                const int64_t rows = (int64_t)(a.tail_slots / 2) * XPB_L;
                ProfScope prof(PROF_DH_MERGE, stream);
                hipLaunchKernelGGL((dh_merge_kernel<D, XPB_L>), dim3((unsigned)((rows + PPB - 1) / PPB)), dim3(256), 0, stream, a);
                e = hipGetLastError();
            }
        }
        if (e == hipSuccess && a.splits > 1) {
            constexpr int PPB = 256 / (D / 8);
            ProfScope prof(PROF_DH_MERGE, stream);
            hipLaunchKernelGGL((dh_merge_kernel<D>), dim3((unsigned)((a.N + PPB - 1) / PPB)), dim3(256), 0, stream, a);
            e = hipGetLastError();
        }
        return e;
    }
    case TILE_PASS_FDH: {  // the dH pass's shapes: same stationary rows, same splits, same last-round plan
        bool done = false;
        if constexpr (XG_B == 2) {
            if (wide(a.N, true)) {
                e = launch_tile_kernel<D, MODE_FDH, BY_B, 4, 2, MINB, NBUF_B>(a, a.N, stream);
                done = true;
            }
        }
        if (!done) e = launch_tile_kernel<D, MODE_FDH, BY_B, NW_L, 1, MINB, NBUF_FDH, DS_B>(a, a.N, stream);
        if constexpr (D > 128) {
            if (e == hipSuccess && a.tail_slots > 0) {
                constexpr int PPB = 256 / (D / 8), XPB_L = NW_L * 32;
                const int64_t rows = (int64_t)(a.tail_slots / 2) * XPB_L;
                ProfScope prof(PROF_FDH_MERGE, stream);
                hipLaunchKernelGGL((fdh_merge_kernel<D, XPB_L>), dim3((unsigned)((rows + PPB - 1) / PPB)), dim3(256), 0, stream, a);
                e = hipGetLastError();
            }
        }
        if (e == hipSuccess && a.splits > 1) {
            constexpr int PPB = 256 / (D / 8);
            ProfScope prof(PROF_FDH_MERGE, stream);
            hipLaunchKernelGGL((fdh_merge_kernel<D>), dim3((unsigned)((a.N + PPB - 1) / PPB)), dim3(256), 0, stream, a);
            e = hipGetLastError();
        }
        return e;
    }
    case TILE_PASS_DE:
        if constexpr (D > 128) {
            // One block of eight wavefronts per compute unit: scatter blocks at the head of this launch would run 256
            // at a time, one long latency chain each, before any tile block starts (c5: 330 us of a 970 us launch).
            // On their own they run many to a compute unit.
            a.scatter_apart = 1;
            if (a.scale_blocks > 0) {  // dH = grad_loss * U wanted as well: next to the scatter, not behind the tiles
                a.scale_blocks = 0;
                if ((e = launch_pos_scatter_scale_d<D>(a, stream)) != hipSuccess) return e;
            } else if ((e = launch_pos_scatter(a, stream)) != hipSuccess) return e;
        }
        if constexpr (XG_B == 2) {
            if (wide(a.n_cols, false)) return launch_tile_kernel<D, MODE_DE, BY_B, 4, 2, MINB, NBUF_B>(a, a.n_cols, stream);
        }
        if (a.filter_log2 > -INFINITY) {
            if constexpr (D > 128) return launch_tile_kernel<D, MODE_DE, BY_B, NW_L, 1, MINB, NBUF_B, DS_B, true>(a, a.n_cols, stream);
            else return hipErrorInvalidValue;
        }
        return launch_tile_kernel<D, MODE_DE, BY_B, NW_L, 1, MINB, NBUF_B, DS_B>(a, a.n_cols, stream);
    default:
        return hipErrorInvalidValue;
    }
}

template <int D>
hipError_t launch_bwd_for_d(TileArgs a_dh, TileArgs a_de, hipStream_t stream)
{
    constexpr int XG_B = (D <= 64) ? 2 : 1;
    a_dh.write_consts = 0;
    if (!a_dh.g_separate) {
        constexpr int PPB = 256 / (D / 8);
        ProfScope prof(PROF_BWD_PRE, stream);
        hipLaunchKernelGGL((bwd_pre_kernel<D>), dim3((unsigned)((a_dh.N + PPB - 1) / PPB)), dim3(256), 0, stream, a_dh);
        const hipError_t pre = hipGetLastError();  // reading the error clears it: read it once
        if (pre != hipSuccess) return pre;
    }
    // two groups of stationary rows per wavefront under the same rule as for the separate launches
    auto wide = [&](int64_t n_x, int splits, bool may_split) {
        const int64_t xb = (n_x + 255) / 256;
        return XG_B == 2 && (xb >= 300 || (may_split && xb < 120 && xb * splits >= 480));
    };
    const bool wide_dh = wide(a_dh.N, a_dh.splits, true), wide_de = wide(a_de.n_cols, a_de.splits, false);
    hipError_t e;
    if (a_dh.filter_log2 > -INFINITY) {  // gradient filtering: one group of stationary rows per wavefront, so that a
        e = launch_bwd_kernel<D, 1, 1, true>(a_dh, a_de, stream);  // dropped block skips a whole second product
    } else if constexpr (XG_B == 2) {
        if (wide_dh && wide_de) e = launch_bwd_kernel<D, 2, 2>(a_dh, a_de, stream);
        else if (wide_dh) e = launch_bwd_kernel<D, 2, 1>(a_dh, a_de, stream);
        else if (wide_de) e = launch_bwd_kernel<D, 1, 2>(a_dh, a_de, stream);
        else e = launch_bwd_kernel<D, 1, 1>(a_dh, a_de, stream);
    } else {
        e = launch_bwd_kernel<D, 1, 1>(a_dh, a_de, stream);
    }
    if (e == hipSuccess && a_dh.splits > 1) {
        constexpr int PPB = 256 / (D / 8);
        ProfScope prof(PROF_DH_MERGE, stream);
        hipLaunchKernelGGL((dh_merge_kernel<D>), dim3((unsigned)((a_dh.N + PPB - 1) / PPB)), dim3(256), 0, stream, a_dh);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kPosChunkApart) void pos_scatter_kernel(TileArgs a)
{
    __shared__ uint64_t keys[kPosChunkApart];
    pos_scatter_block<D, kPosChunkApart>(a, blockIdx.x, keys);
}

// The correct-item scatter and the scaling dH = grad_loss * U in one launch (hidden size 256, where neither rides in
// the dE launch): the scatter is bound by latencies and atomics, the scaling by memory bandwidth, and they share no
// data, so side by side they take about as long as the scatter alone.  The scaling blocks also file grad_loss under the
// compacted index for the dE pass that follows.
template <int D>
__global__ __launch_bounds__(kPosChunkApart) void pos_scatter_scale_kernel(TileArgs a, int64_t scatter_blocks)
{
    __shared__ uint64_t keys[kPosChunkApart];
    if ((int64_t)blockIdx.x < scatter_blocks) {
        pos_scatter_block<D, kPosChunkApart>(a, blockIdx.x, keys);
        return;
    }
    const int64_t chunk = ((int64_t)blockIdx.x - scatter_blocks) * kPosChunkApart + threadIdx.x;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    if (chunk < n_pos) a.de_const[a.N + chunk] = __float_as_uint(a.g ? a.g[pos_row(a, chunk)] : 1.f);
    dh_scale_chunk<D>(a, chunk);
}

template <int D>
hipError_t launch_pos_scatter_scale_d(const TileArgs &a, hipStream_t stream)
{
    if (a.N == 0) return hipSuccess;
    const int64_t scatter_blocks = (a.N + kPosChunkApart - 1) / kPosChunkApart;
    const int64_t scale_blocks = (a.N * (D / 8) + kPosChunkApart - 1) / kPosChunkApart;
    ProfScope prof(PROF_POS_SCATTER, stream);
    hipLaunchKernelGGL((pos_scatter_scale_kernel<D>), dim3((unsigned)(scatter_blocks + scale_blocks)), dim3(kPosChunkApart), 0, stream, a,
                       scatter_blocks);
    return hipGetLastError();
}

template <int D>
hipError_t launch_dh_scale_d(const TileArgs &a, bool file_g, hipStream_t stream)
{
    if (a.N == 0) return hipSuccess;
    const dim3 grid((unsigned)((a.N * (D / 8) + 255) / 256)), block(256);
    ProfScope prof(PROF_DH_SCALE, stream);
    if (file_g) hipLaunchKernelGGL((dh_scale_kernel<D, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((dh_scale_kernel<D, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int D>
hipError_t launch_pos_scatter_d(const TileArgs &a, hipStream_t stream)
{
    if (a.N == 0) return hipSuccess;
    const dim3 grid((unsigned)((a.N + kPosChunkApart - 1) / kPosChunkApart)), block(kPosChunkApart);
    ProfScope prof(PROF_POS_SCATTER, stream);
    hipLaunchKernelGGL((pos_scatter_kernel<D>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace cce
