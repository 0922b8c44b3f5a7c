/*
 * cce_neg.h - C ABI of the fused cross-entropy loss with negative sampling (CCE-)
 * for AMD MI355X (gfx950).
 *
 * The operation is the paper's Sec. 3.3 ("Cut-Cross-Entropy with Negative
 * Sampling"): for every position i of the flattened final-layer output H [N,d]
 * (the paper's E), score it against its correct item and K sampled negative items
 * taken from the item table E [V,d] (the paper's classifier C, stored row-major
 * as C^T), and return
 *
 *     lse_i  = log sum_j exp(<H_i, E_{c_ij}>)         (Eq. 5, indexed log-sum-exp)
 *     loss_i = lse_i - <H_i, E_{tgt_i}>               (Eq. 4, per position, l = o+ - LSE, L = -mean l)
 *
 * without ever writing the [N x (K+1)] score matrix to device memory (Alg. 1).
 * The backward call recomputes the scores, forms the softmax S = exp(o - LSE)
 * and returns dH and the scatter-added dE (Eq. 6, Alg. 2), folding in the
 * gradient of the correct-item score (the first term of Eq. 4).  The
 * full-catalogue mode is the paper's Sec. 3.1 loss (Eq. 2): all V items are the
 * candidates, no sampling, no gradient filtering.
 *
 * All pointers are DEVICE pointers owned by the caller, row-major, contiguous and
 * 16-byte aligned.  The library allocates and frees nothing.  Work is enqueued on
 * the HIP stream passed in (hipStream_t as void*, NULL = default stream) and the
 * calls return without synchronising.  Scalars of the mean reduction (Eq. 3) are
 * the caller's business: pass grad_loss[i] = 1/N_valid for a mean loss.
 */
#ifndef CCE_NEG_H
#define CCE_NEG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CCE_OK = 0,
    CCE_ERR_NULL = 1,        /* a required pointer is NULL */
    CCE_ERR_SHAPE = 2,       /* N < 0, V <= 0, K < 0, d not a multiple of 8 in [8,512], V or K beyond int32 */
    CCE_ERR_DTYPE = 3,       /* unknown dtype, or dH_dtype = BF16 with fp32 inputs */
    CCE_ERR_INDEX = 4,       /* an id of a valid position was outside [0,V) (reported by cce_neg_index_status) */
    CCE_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or smaller than cce_neg_workspace_bytes() */
    CCE_ERR_UNSUPPORTED = 6, /* the requested algo cannot run this descriptor */
    CCE_ERR_HIP = 7          /* a HIP runtime call (launch) failed */
} cce_status;

typedef enum { CCE_F32 = 0, CCE_BF16 = 1 } cce_dtype;

typedef enum {
    CCE_NEG_SHARED = 0,       /* neg is [K]: one list of negatives for all positions */
    CCE_NEG_PER_POSITION = 1, /* neg is [N,K]: row i holds the negatives of position i (the paper's Inds without its first column) */
    CCE_NEG_FULL = 2          /* neg ignored: all V items are candidates (Sec. 3.1, Eq. 2) */
} cce_neg_mode;

typedef enum {
    CCE_ALGO_AUTO = 0,   /* library picks: MFMA tiles for bf16 shared/full, row gathers otherwise */
    CCE_ALGO_GATHER = 1, /* one wavefront per position, candidate rows gathered one by one (Alg. 1 / Alg. 2 as printed) */
    CCE_ALGO_TILE = 2    /* dense H x E_neg^T score tiles on the matrix cores; bf16 inputs, shared or full mode only */
} cce_algo;

typedef struct {
    int64_t N;                      /* positions = batch * sequence length (Sec. 3.1) */
    int64_t V;                      /* catalogue size, rows of E */
    int32_t d;                      /* hidden size; multiple of 8, 8..512; never split (Sec. 3.3) */
    int32_t K;                      /* negatives per position (the paper's ns); ignored for CCE_NEG_FULL; 0 allowed */
    int32_t in_dtype;               /* cce_dtype of H and E */
    int32_t dH_dtype;               /* cce_dtype of dH: F32, or BF16 (round-to-nearest-even) when in_dtype is BF16 */
    int32_t neg_mode;               /* cce_neg_mode */
    int32_t mask_target_collisions; /* 1: a negative equal to the position's own target is left out of LSE and gradients */
    int32_t validate_indices;       /* 1: kernels range-check ids of valid positions, never dereference bad ones and raise the
                                       status word (see cce_neg_index_status for what a flagged call returns) */
    int32_t algo;                   /* cce_algo */
    int32_t reuse_forward_prep;     /* backward only, 1: the caller vouches that the workspace still holds what the
                                       forward call with this descriptor and the same tgt / neg / mask contents left
                                       there (nothing else wrote to it since: no other forward call, no backward call
                                       without this flag; backward calls with it may repeat), so the compaction of
                                       padded positions,
                                       the collision counts and (hidden sizes up to 128, grad_loss given) the
                                       per-position constants that the forward call files for the backward pass are
                                       not recomputed; lse must then be the forward call's own output.  0: no
                                       assumption.  With 1 and a workspace that does not hold them the results are
                                       undefined. */
    float filter_eps;               /* backward only, gradient filtering of the full-catalogue mode (Sec. 3.1, last
                                       paragraph; threshold sweep: Sec. 5, "Gradient Filtering with CCE", and the
                                       appendix "Sparsity Threshold Analysis"): 0 = off.  > 0: the softmax matrix of the valid positions
                                       (batch order) by the items (id order) is cut into 32 x 32 blocks aligned at the
                                       origin, and a block whose largest probability is below filter_eps counts as
                                       zero in Eq. 6 (it adds nothing to dH or dE; the term of the correct item stays).
                                       loss and lse are exact.  Needs CCE_NEG_FULL, bf16 inputs and d in {64,128,256},
                                       else CCE_ERR_UNSUPPORTED; negative or NaN: CCE_ERR_SHAPE. */
    int32_t fuse_dH;                /* 1: the forward call also forms the hidden-state gradient short of the upstream
                                       gradient, U_i = sum_j softmax_ij E_cij - E_tgt_i (Eq. 6 left with grad LSE = 1 and the
                                       correct item's term), in the same pass over the candidates that yields lse (an
                                       online softmax: no log-sum-exp is known yet, the rows are divided by the sum at the
                                       end), and keeps it in the workspace (4 N d bytes more); a backward call with this
                                       flag AND reuse_forward_prep = 1 then writes dH_i = grad_loss_i U_i and computes the
                                       scores once more for dE only: four products of the size of the score matrix per
                                       step instead of five, two exponentials per score instead of three.  Set it the
                                       same way in the size query, the forward and the backward descriptor.  On the
                                       row-gather kernels (fp32, other hidden sizes, per-position negatives) the forward
                                       call sums the weighted candidate rows while it has them in registers for the
                                       score, and the backward call gathers no candidate row for dH (same 4 N d bytes).
                                       Ignored for per-position negatives beyond the inverted index (2^31 pairs and
                                       more), and by a backward call without reuse_forward_prep or with filter_eps > 0
                                       (those run the dH pass as without the flag).  A forward-only caller leaves it 0. */
} cce_desc;

/* Bytes of device workspace both calls need for this descriptor.  Returns 0 for an invalid descriptor.
 *   shared / full mode, bf16:  20 bytes per position (compaction, collision counts, coefficients), 4 d more with fuse_dH,
 *                              plus partial
 *                              results of split launches: 8 bytes per position and forward split, and, for batches
 *                              of at most 40,960 positions, 4 d bytes per position and dH split; hidden size 256 and
 *                              more than 65,536 positions: 64 MiB of partial dH rows for the split of the last round
 *                              of blocks;
 *   per-position mode:         the inverted index that turns the dE scatter into a gather (pairs sorted by item) is
 *                              built and used up in slices of the item-id range: 12 1/8 bytes per pair of ONE slice,
 *                              a slice holding at most B = max(2^22, N K / 8) pairs (so at most 51 MB up to
 *                              N K = 2^25 pairs, and 3/8 of the bytes of the [N,K] id matrix itself beyond), plus
 *                              4 bytes per table row, 4 per position and at most 32 MiB of bucket counts.  Catalogues
 *                              of more than 2^22 items whose pairs exceed B: a 256-byte header (they keep the atomic
 *                              row adds of Alg. 2);
 *   otherwise:                 a 256-byte header (with fuse_dH: 4 + 4 d bytes per position more, also in per-position mode);
 *   shared mode, in addition:  4 bytes per negative (where the *_sampled calls write the list they draw).
 * No score, probability or gradient-coefficient matrix is ever stored: the workspace holds indices and per-position
 * scalars only.  The same workspace may be reused by later calls on the same stream. */
size_t cce_neg_workspace_bytes(const cce_desc *desc);

/* Clears the workspace header (index status word).  Call once after allocating a workspace, on the stream that will
 * use it; enqueues a small fill kernel (no memset node, so it is safe under stream capture). */
cce_status cce_neg_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward (Alg. 1; Eq. 4, Eq. 5).
 *   H     [N,d]  in_dtype          hidden states
 *   E     [V,d]  in_dtype          item table
 *   tgt   [N]    int32             correct item per position (first column of the paper's Inds)
 *   neg   [K] or [N,K] int32       negatives (NULL allowed when K == 0 or mode FULL); duplicates count once each
 *   mask  [N]    uint8, nullable   1 = valid, 0 = padding; NULL = all valid.  For a padded position loss = lse = +0
 *                                  and its tgt / neg entries are never read.
 *   loss  [N]    float  (out)      lse_i - o+_i, fully overwritten
 *   lse   [N]    float  (out)      fully overwritten; feed it to cce_neg_backward
 * Host-checkable errors are returned before anything is launched and nothing is written.
 */
cce_status cce_neg_forward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                           const uint8_t *mask, float *loss, float *lse, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/*
 * Backward (Alg. 2; Eq. 6; S = exp(o - LSE)).
 *   lse        [N] float            from the forward call on the same inputs
 *   grad_loss  [N] float, nullable  upstream gradient of loss_i (the paper's grad LSE); NULL = 1
 *   dH  [N,d] dH_dtype (out)        fully overwritten, rows of padded positions are zero
 *   dE  [V,d] float (in/out)        ACCUMULATED INTO (floating-point atomics, or one read-modify-write per row in
 *                                   per-position mode): the caller zeroes it or carries earlier gradients; rows that
 *                                   no valid position indexes are left untouched
 * With G_ij = grad_loss_i * (softmax_ij - [j is the correct item]):
 *   dH_i = sum_j G_ij E_{c_ij},   dE_{c_ij} += G_ij H_i.
 */
cce_status cce_neg_backward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                            const uint8_t *mask, const float *lse, const float *grad_loss, void *dH, float *dE,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * cce_neg_forward for callers that can hand over no workspace and must not allocate: code under HIP graph capture,
 * tight serving loops (scoring a batch needs the forward pass only), harnesses that forbid allocation.  Same inputs,
 * outputs and results as cce_neg_forward; the scratch memory the kernels need (compaction of padded positions,
 * collision counts, partial max / sum of split launches) lives in a fixed array inside the library's code object,
 * CCE_NEG_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends.  Nothing is allocated or freed by the call:
 * the array's device address is looked up once per device (hipGetSymbolAddress, on the first call with that device
 * current; make that first call outside a graph capture) and a small fill kernel clears the array's header, which
 * keeps whatever the last call left there.
 *   - A descriptor whose forward pass needs more scratch than the array holds is refused with CCE_ERR_WORKSPACE
 *     before anything is launched.  Matrix-core path: 20 bytes per position, plus 8 per position and split where the
 *     candidate range is split (at most 8 ways), so 32 MiB carry between 390,000 and 1,600,000 positions; other
 *     paths need 256 bytes.  validate_indices = 1 is refused with CCE_ERR_UNSUPPORTED (there is no status
 *     word the caller could read).
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads) race.
 *     Calls on one stream are ordered and safe.
 *   - A backward call cannot reuse what this call left (reuse_forward_prep needs a caller-owned workspace).
 */
#define CCE_NEG_NOALLOC_SCRATCH_BYTES (32u << 20)
cce_status cce_neg_forward_noalloc(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt,
                                   const int32_t *neg, const uint8_t *mask, float *loss, float *lse, void *hip_stream);

/*
 * Negative sampling inside the kernels.  The paper draws the negatives of a step on the host (global uniform sampling,
 * or popularity-based sampling through a multinomial over the catalogue: Sec. 5, "Comparison Sampling Strategies")
 * and names the stored index matrix as the memory cost of CCE- over CCE (Sec. 5, "What is better").  The *_sampled
 * calls take a sampler instead of `neg`: every id is a pure function of (seed, stream, position, slot), recomputed
 * wherever the kernels need it, so the [N,K] matrix is never stored (the backward call's inverted index holds one
 * slice of (item, position) pairs at a time, see cce_neg_workspace_bytes).
 *   generator  Philox4x32-10 (Salmon et al., SC'11), key = (seed low word, seed high word),
 *              counter = (q, position low word, position high word, stream)
 *   slot s (0 <= s < K) of position i is draw j = s + 1
 *   UNIFORM    q = j >> 2, r = output word j & 3, id = floor(r V / 2^32)
 *   ALIAS      q = j >> 1, (r0, r1) = output words 2(j & 1), 2(j & 1) + 1, c = floor(r0 V / 2^32),
 *              id = r1 < alias_thresh[c] ? c : alias_id[c]     (alias method; the caller builds the table for its law)
 *   CCE_NEG_SHARED uses the draws of position 0 for every position.
 * Draws are independent (sampling with replacement): repeated ids count once each, an id equal to the position's own
 * target is handled by mask_target_collisions as for stored negatives.  Change `stream` (or the seed) every step.
 */
typedef enum { CCE_SAMPLER_UNIFORM = 1, CCE_SAMPLER_ALIAS = 2 } cce_sampler_kind;

typedef struct {
    int32_t kind;                 /* cce_sampler_kind */
    uint32_t stream;              /* fourth counter word: e.g. the training step */
    uint64_t seed;                /* generator key */
    const uint32_t *alias_thresh; /* DEVICE [V], ALIAS only: column c keeps id c with probability alias_thresh[c] / 2^32 */
    const int32_t *alias_id;      /* DEVICE [V], ALIAS only: the id column c yields otherwise; must lie in [0,V) */
} cce_sampler;

/* Writes the ids the sampler denotes for this descriptor: neg_out [K] (CCE_NEG_SHARED) or [N,K] (CCE_NEG_PER_POSITION,
 * all positions, padded ones included), DEVICE int32, fully overwritten.  For inspection and tests; the *_sampled
 * calls do not need it.  CCE_NEG_FULL: CCE_ERR_UNSUPPORTED.  Unknown kind: CCE_ERR_SHAPE.  Missing table: CCE_ERR_NULL. */
cce_status cce_neg_sample(const cce_desc *desc, const cce_sampler *sampler, int32_t *neg_out, void *hip_stream);

/* cce_neg_forward / cce_neg_backward with neg replaced by the sampler; every other argument, output and error as
 * there.  Results equal those of the plain calls on the ids cce_neg_sample writes.  Per-position mode: ids of padded
 * positions are never generated, the forward pass, the backward pass and the index build of the dE pass draw them
 * again.  Shared mode: the K ids are written to a reserved corner of the workspace first.  Pass the same sampler to
 * the backward call as to the forward call. */
cce_status cce_neg_forward_sampled(const cce_desc *desc, const cce_sampler *sampler, const void *H, const void *E,
                                   const int32_t *tgt, const uint8_t *mask, float *loss, float *lse, void *workspace,
                                   size_t workspace_bytes, void *hip_stream);
cce_status cce_neg_backward_sampled(const cce_desc *desc, const cce_sampler *sampler, const void *H, const void *E,
                                    const int32_t *tgt, const uint8_t *mask, const float *lse, const float *grad_loss,
                                    void *dH, float *dE, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Synchronises hip_stream and reads the index status word kept in workspace.  Returns CCE_ERR_INDEX if any call on
 * that workspace since the last query found an id outside [0,V) on a valid position (validate_indices = 1 only),
 * CCE_OK otherwise; the word is cleared.  Bad ids are never dereferenced.  Row-gather kernels (per-position mode, fp32
 * inputs, CCE_ALGO_GATHER): a bad negative is skipped and a position with a bad target is treated as padding, so the
 * outputs are those of the sanitised problem.  Matrix-core kernels (bf16 shared / full mode): a position with a bad
 * target is treated as padding, but a bad SHARED negative is scored as item 0 in its place; the outputs of a flagged
 * call are then unspecified (finite, in bounds, and dE row 0 may have received gradient): discard them.
 */
cce_status cce_neg_index_status(void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Measurement aid for benchmarks and profilers (not part of the method).  While enabled, every kernel launch the library
 * makes is bracketed by a pair of HIP events on the launch stream.  cce_neg_profile_read waits for the recorded events,
 * adds the elapsed time per kernel family and returns the number of families written (at most max):
 *   names     [max][32] char (HOST)   family name, NUL-terminated: "gather_fwd", "gather_bwd", "prep", "tile_fwd",
 *                                     "fwd_merge", "tile_dh", "dh_merge", "tile_de", "index", "item_de", "pos_scatter",
 *                                     "bwd_pre", "tile_bwd" (dH and dE pass in one launch)
 *   total_ms  [max] float (HOST)      summed duration since the last read
 *   launches  [max] int32 (HOST)      launches since the last read
 * The records are cleared by the read.  Enabling creates HIP events on demand; nothing else in the library allocates.
 * Not thread-safe; leave it disabled in production.
 */
cce_status cce_neg_profile_enable(int32_t enable);
int32_t cce_neg_profile_read(int32_t max, char *names, float *total_ms, int32_t *launches);

/* Static, NUL-terminated description of a status code. */
const char *cce_status_string(cce_status status);

#ifdef __cplusplus
}
#endif
#endif /* CCE_NEG_H */
