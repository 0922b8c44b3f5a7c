// Host-side launch entry points of the kernel families and their argument blocks (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include "cce_device.hpp"

namespace cce {

// 32-bit words of the workspace header.
enum { kHdrStatus = 0, kHdrTotal = 1, kHdrDone = 2, kHdrNValid = 3, kHdrHot = 4 };

// ---- row-gather family: one wavefront per position; any mode, fp32 or bf16 inputs
hipError_t launch_gather(bool backward, bool bf16, const Params &p, hipStream_t stream);
// dE of the negatives shared by all positions (shared list or full catalogue), candidate-major; row-gather family
hipError_t launch_shared_dE(bool bf16, const Params &p, hipStream_t stream);
// backward side of the fused forward pass of the row-gather family (Params::U set by the forward call): dH = grad_loss * U,
// and with pos_rows the correct items' dE rows by atomics
hipError_t launch_gather_scale(bool bf16, bool pos_rows, const Params &p, hipStream_t stream);

// ---- matrix-core family: bf16 inputs, shared negatives or full catalogue
struct PrepArgs {
    const int32_t *tgt;
    const int32_t *neg;    // shared negatives [K] or nullptr
    const uint8_t *mask;   // nullable
    int32_t *header;       // workspace header words
    int32_t *idx;          // out: compacted valid positions (nullptr: no compaction wanted)
    int32_t *cnt;          // out: multiplicity of the target among the negatives (nullptr: not wanted)
    float *loss, *lse;     // forward: zeroed for padded positions (nullable)
    int64_t N, V;
    int32_t d, K, validate, dH_bf16;
};

struct TileArgs {
    const uint16_t *H;
    const uint16_t *E;
    const int32_t *tgt;
    const int32_t *neg;          // candidate column -> item row; nullptr = identity (full catalogue)
    const int32_t *idx;          // compacted position -> position row; nullptr = identity
    const int32_t *n_valid_ptr;  // device count of valid positions; nullptr = N
    const int32_t *cnt;          // target multiplicity per position; nullptr = 0
    const uint8_t *pos_mask;     // stand-alone scatter without compaction: padding mask (nullable)
    const float *lse_in;
    const float *g;
    float *loss, *lse;
    void *dH;
    float *dE;
    float *coef;                 // [N] coefficient of the correct item, written by the dH pass, read by the scatter
    uint32_t *de_const;          // [2, N] per compacted position (float bits): exponent offset -lse log2e and upstream
                                 // gradient g of the dE coefficient; written ahead of the dE pass, streamed by it
    float *U;                    // [N, d] fused forward pass (out), dH scaling (in): the hidden-state gradient short of the
                                 // upstream gradient, U_i = sum_j p_ij E_cij - E_tgt_i, filed under the position's row
    float *part_m, *part_s;      // [splits, N] partial max / sum of split forward runs
    float *part_dH;              // [splits, N, d] partial dH of split runs
    int64_t N, V, n_cols;        // n_cols = K, or V in full-catalogue mode
    int64_t pos_blocks;          // dE launch: blocks [0, pos_blocks) scatter the correct items, the rest run the dE pass
    int64_t pad_blocks;          // dH launch: blocks [0, pad_blocks) zero the dH rows of padded positions (set by the launcher)
    int64_t scale_block0;        // dE launch: blocks from this one on write dH = grad_loss * U (set by the launcher; none
                                 // when scale_blocks is 0)
    int64_t scale_blocks;
    int32_t d, splits, pos_weight_mode, dH_bf16, validate;  // splits: upper bound on entry to launch_tile, chosen factor inside
    int32_t write_consts;        // dH pass: 1 = it files coef and de_const itself (dE launched after it), 0 = a pass before it did
    float filter_log2;           // backward, gradient filtering: log2 of the threshold; -inf = off
    int32_t scatter_apart;       // dE launch: 1 = the correct-item scatter has been launched on its own, no leading blocks here
    int32_t tail_slots;          // dH pass, > 0: blocks the chip holds at once; the position blocks of the last, partly filled
                                 // round split the candidate range among the idle block slots (planned on the device from
                                 // the count of valid positions), partial rows in part_dH, summed by the tail merge
    int32_t g_stream_off;        // dE pass with g_separate: 1 = grad_loss is NOT streamed by row number but read from the second
                                 // half of de_const, where a pass before this one filed it under the compacted index
    int32_t g_separate;          // backward: coef and de_const[0] are what the FORWARD pass left (no upstream gradient in
                                 // them): the scatter multiplies by g itself and the dE pass streams g by row number
};

// The dE launch also scatters the correct items.  FDH: forward pass that also forms U (TileArgs::U) with an online softmax.
enum { TILE_PASS_FWD = 0, TILE_PASS_DH = 1, TILE_PASS_DE = 2, TILE_PASS_FDH = 3 };
// dH = grad_loss * U for valid positions, zero rows for padded ones, as a launch of its own; with file_g the upstream
// gradient is also filed under the compacted index (second half of de_const) for a dE pass that does not stream it by row.
hipError_t launch_dh_scale(const TileArgs &a, bool file_g, hipStream_t stream);
// dH and dE passes in one launch (hidden sizes up to 128): a_dh.splits / a_de.splits carry the two split bounds.
bool tile_backward_fusable(int d);
hipError_t launch_tile_backward(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream);

// ---- inverted-index dE of per-position negatives
struct InvertArgs {
    const void *H;
    const void *E;
    const int32_t *tgt;
    const int32_t *neg;      // [N,K]
    const uint8_t *mask;     // nullable
    const float *lse_in;
    const float *g;          // nullable
    float *dE;
    int32_t *cursor;         // [V] workspace: counts -> segment starts -> segment ends
    int32_t *block_sums;     // [invert_scan_blocks(V)] workspace
    int32_t *pairs;          // [invert_index_pairs] workspace: positions filed under their item (of the slice at hand)
    int2 *tmp;               // [invert_index_pairs] workspace: (id, position) partitioned by bucket (of the slice at hand)
    int32_t *bucket_start;   // [n_buckets] workspace: where a bucket starts in the arrays of its slice (nullptr: unsliced)
    int32_t *slice_of;       // [n_buckets] workspace: slice of every bucket, -1 = out of the index (nullptr: unsliced)
    int32_t *slice_hot;      // [invert_plan_words] workspace: per slice the work-list counter, first and last bucket; a flag
    int64_t budget, n_chunks;  // pairs per slice at most; chunks of 8192 pairs in all
    int32_t n_slices, slice;   // slices of this call; the one this launch works on
    int32_t *part_hist;      // [n_buckets * n_part_blocks + 1] workspace: (bucket, block) counts -> offsets
    int32_t *part_total;     // = part_hist + n_buckets * n_part_blocks (set by the launcher)
    int4 *hot_list;          // [hot_capacity] workspace: (item, first pair, end pair, -) chunks of items with long segments
    int32_t *hot_count;      // workspace header word: chunks filed
    int32_t hot_capacity;
    int64_t N, V, n_part_blocks;
    int32_t d, K, collide, validate, n_buckets;
    Sampler smp;             // kind != 0: the negatives are drawn again here instead of being read from neg
};
size_t invert_hot_capacity(int64_t N, int64_t K);  // entries of hot_list
int64_t invert_pair_budget(int64_t N, int64_t K);  // pairs one slice of the index holds at most
int64_t invert_index_pairs(int64_t N, int64_t K);  // entries of pairs / tmp: min(N K, budget)
int invert_slices(int64_t N, int64_t K);           // slices of the item-id range the index is built in
int invert_plan_words();                           // words of slice_hot
size_t invert_scan_blocks(int64_t n);          // blocks of the scan over n words (size of block_sums)
int64_t invert_part_blocks(int64_t N, int64_t K);
int64_t invert_buckets(int64_t V);
bool invert_partitioned(int64_t V);            // false: catalogue too large for the LDS bucket histogram, atomics are used
// scatter != nullptr: the correct items' gradient rows are scattered on the way (their blocks lead the second index pass)
hipError_t launch_inverted_dE(bool bf16, const InvertArgs &a, const TileArgs *scatter, hipStream_t stream);

// Aggregated scatter of the correct items on its own (bf16 inputs, d in {64,128,256}): dE[tgt_i] += coef_i * H_i.
hipError_t launch_pos_scatter(const TileArgs &a, hipStream_t stream);

bool tile_supports_d(int d);
size_t tile_tail_partial_bytes(int64_t N, int d);  // partial dH rows of the last-round split (0: not used for this shape)
hipError_t launch_prep(const PrepArgs &p, hipStream_t stream);
hipError_t launch_tile(int pass, const TileArgs &a, hipStream_t stream);

// Event bracket around a kernel launch while profiling is enabled (see cce_neg_profile_enable); otherwise a no-op.
enum { PROF_GATHER_FWD = 0, PROF_GATHER_BWD, PROF_PREP, PROF_TILE_FWD, PROF_FWD_MERGE, PROF_TILE_DH, PROF_DH_MERGE,
       PROF_TILE_DE, PROF_INDEX, PROF_ITEM_DE, PROF_POS_SCATTER, PROF_BWD_PRE, PROF_TILE_BWD, PROF_TILE_FDH, PROF_FDH_MERGE,
       PROF_DH_SCALE, PROF_FAMILIES };
struct ProfScope {
    ProfScope(int family, hipStream_t stream);
    ~ProfScope();
    int slot;
    hipStream_t stream;
};

// Writes the ids a sampler denotes: out[n_pos, K], row i = draws 1..K of position i (n_pos = 1: the shared list).
hipError_t launch_sample(const Sampler &smp, int64_t n_pos, int32_t K, int32_t *out, hipStream_t stream);

// Clears `words` 32-bit words at dst with a fill kernel (no memset node).
hipError_t launch_fill_zero(int32_t *dst, size_t words, hipStream_t stream);

}  // namespace cce
