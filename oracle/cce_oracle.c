/*
 * fp64 CPU oracle for the cross-entropy loss with negative sampling (CCE-).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the loss
 * computes, written from the paper's equations, one position at a time, in
 * double precision, two-pass (max, then sum of exponentials), with no blocking,
 * fusion or reordering.  It shares no code with the GPU library and nothing in
 * the product path may call it; only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.
 *
 * What is computed, for every selected valid position i (paper notation in
 * brackets; the paper calls the hidden states E and the classifier C, here they
 * are H [N,d] and the item table E [V,d]):
 *
 *   candidates   c_0 = tgt_i (the correct item, "j = 1" in Sec. 3.3), then the
 *                K negatives (shared list, or row i of the per-position matrix);
 *                in full-catalogue mode the candidates are all V ids once and
 *                the correct item is the candidate whose id equals tgt_i.
 *   scores       o_j   = <H_i, E_{c_j}>                      (Alg. 1, scalar product)
 *   LSE          lse_i = log sum_{live j} exp(o_j)           (Eq. 5)
 *   loss         loss_i = lse_i - o_pos                      (Eq. 4: l = o+ - LSE, L = -mean l)
 *   softmax      p_j   = exp(o_j - lse_i)                    (S = exp(o - LSE), Sec. 3.3)
 *   coefficient  G_j   = g_i * (p_j - [j is the correct item])
 *   gradients    dH_i  = sum_j G_j * E_{c_j}                 (Eq. 6, left)
 *                dE_{c_j} += G_j * H_i                       (Eq. 6, right; Alg. 2 indexed update)
 *
 * G folds the two gradient paths the paper keeps apart (the LSE kernel, scaled
 * by the upstream gradient of LSE, and the correct-logit kernel): with
 * loss = lse - o+, d loss/d lse = +g and d loss/d o+ = -g.
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - a candidate is "live" unless it is a negative whose id equals the
 *     position's own target and mask_collisions is set; dead candidates add
 *     nothing to LSE or to any gradient;
 *   - negatives are a multiset: a repeated id counts once per occurrence;
 *   - masked positions (mask[i]==0) give loss = lse = 0, dH row = 0, no dE
 *     contribution, and their ids are never read;
 *   - K = 0 gives loss = 0 and zero gradients (p of the only candidate is 1).
 *
 * Gradient filtering (Sec. 3.1, last paragraph: computations with values below a
 * prescribed threshold are disregarded in the backward pass; Sec. 3.3 notes that it
 * can follow step 4 of Alg. 2; Sec. 5, "Gradient Filtering with CCE", and the appendix
 * "Sparsity Threshold Analysis" sweep the threshold filter_eps).  The paper
 * gives no granularity.  Reading taken here: the softmax matrix of the valid
 * positions (batch order) by the candidates (catalogue order) is cut into square
 * blocks of `block` entries a side, aligned at the origin; a block whose largest
 * probability is below filter_eps is taken as zero in Eq. 6, the subtraction of
 * the one-hot target stays.  loss and lse are not touched.  cce_oracle_filter_blocks
 * marks the surviving entries, cce_oracle_run applies the marks (p_keep).
 *
 * Parity pins: the tests under tests/ (marker "not gpu") check this file against
 * brute-force full softmax, the K = V-1 full-catalogue identity, central finite
 * differences, closed forms (H = 0, dominant score), softmax rows summing to 1,
 * the zero column sum of dE, random partitions of the candidates merged pairwise (the
 * identity behind Alg. 1), sparse matrix products for Eq. 6, and
 * torch's fp64 logsumexp / autograd on explicitly gathered logits.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_NEG_SHARED = 0, ORACLE_NEG_PER_POSITION = 1, ORACLE_NEG_FULL = 2 };

/* Exact widening of one stored element to double. */
static inline double load_elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int cce_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Runs forward and backward for the positions listed in sel[0..n_sel) (sel NULL:
 * all N positions, n_sel ignored).  Output row r belongs to position sel[r].
 *
 *   loss, lse : [n_out] double, always written
 *   dH        : [n_out, d] double, written when non-NULL
 *   dE        : accumulated into when non-NULL.  With row_slot NULL it is dense
 *               [V, d]; otherwise row_slot[v] is the row of dE that receives
 *               updates of item v (every touched item must have a slot >= 0,
 *               else the function returns 3).
 *   p_out     : [n_out, n_cand] softmax values (0 for dead candidates), optional;
 *               n_cand = K+1 for the sampled modes, V for the full catalogue
 *   g         : [N] upstream gradient per position, NULL = 1
 *   p_keep    : [n_out, n_cand] bytes, optional: where 0, the softmax value counts
 *               as zero in the gradients (gradient filtering); p_out still holds
 *               the unfiltered softmax
 *
 * Returns 0, 1 (bad argument), 2 (id out of range), 3 (missing dE slot).
 */
int cce_oracle_run(int64_t N, int64_t V, int32_t d, int32_t K, int32_t in_dtype, int32_t neg_mode,
                   int32_t mask_collisions, const void *H, const void *E, const int32_t *tgt,
                   const int32_t *neg, const uint8_t *mask, const double *g, int64_t n_sel,
                   const int64_t *sel, double *loss, double *lse, double *dH, const int64_t *row_slot,
                   double *dE, double *p_out, const uint8_t *p_keep)
{
    if (N < 0 || V <= 0 || d <= 0 || K < 0 || !H || !E || !tgt || !loss || !lse)
        return 1;
    if (neg_mode != ORACLE_NEG_FULL && K > 0 && !neg)
        return 1;
    const int64_t n_out = sel ? n_sel : N;
    const int64_t n_cand = (neg_mode == ORACLE_NEG_FULL) ? V : (int64_t)K + 1;
    int status = 0;

#pragma omp parallel
    {
        double *o = (double *)malloc(sizeof(double) * (size_t)n_cand);
        double *h = (double *)malloc(sizeof(double) * (size_t)d);
        double *dh = (double *)malloc(sizeof(double) * (size_t)d);
        int64_t *cand = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_cand);
        unsigned char *live = (unsigned char *)malloc((size_t)n_cand);

#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < n_out; ++r) {
            const int64_t i = sel ? sel[r] : r;
            if (i < 0 || i >= N) {
#pragma omp atomic write
                status = 1;
                continue;
            }
            if (mask && mask[i] == 0) {
                loss[r] = 0.0;
                lse[r] = 0.0;
                if (dH)
                    for (int t = 0; t < d; ++t)
                        dH[r * d + t] = 0.0;
                if (p_out)
                    for (int64_t j = 0; j < n_cand; ++j)
                        p_out[r * n_cand + j] = 0.0;
                continue;
            }
            const int64_t ti = tgt[i];
            int bad = (ti < 0 || ti >= V);
            int64_t pos = 0;

            /* candidate list and liveness */
            if (neg_mode == ORACLE_NEG_FULL) {
                for (int64_t j = 0; j < V; ++j) {
                    cand[j] = j;
                    live[j] = 1;
                }
                pos = ti;
            } else {
                cand[0] = ti;
                live[0] = 1;
                for (int64_t j = 1; j <= K; ++j) {
                    const int64_t id = (neg_mode == ORACLE_NEG_SHARED) ? neg[j - 1] : neg[i * (int64_t)K + (j - 1)];
                    if (id < 0 || id >= V)
                        bad = 1;
                    cand[j] = id;
                    live[j] = !(mask_collisions && id == ti);
                }
                pos = 0;
            }
            if (bad) {
#pragma omp atomic write
                status = 2;
                continue;
            }

            for (int t = 0; t < d; ++t)
                h[t] = load_elem(H, in_dtype, i * (int64_t)d + t);

            /* scores */
            for (int64_t j = 0; j < n_cand; ++j) {
                double s = 0.0;
                for (int t = 0; t < d; ++t)
                    s += h[t] * load_elem(E, in_dtype, cand[j] * (int64_t)d + t);
                o[j] = s;
            }

            /* log-sum-exp over live candidates, two passes */
            double m = -INFINITY;
            for (int64_t j = 0; j < n_cand; ++j)
                if (live[j] && o[j] > m)
                    m = o[j];
            double sum = 0.0;
            for (int64_t j = 0; j < n_cand; ++j)
                if (live[j])
                    sum += exp(o[j] - m);
            const double l = m + log(sum);
            lse[r] = l;
            loss[r] = l - o[pos];

            /* softmax, coefficients, gradients */
            const double gi = g ? g[i] : 1.0;
            for (int t = 0; t < d; ++t)
                dh[t] = 0.0;
            for (int64_t j = 0; j < n_cand; ++j) {
                const double p = live[j] ? exp(o[j] - l) : 0.0;
                if (p_out)
                    p_out[r * n_cand + j] = p;
                if (!live[j])
                    continue;
                const double pf = (p_keep && !p_keep[r * n_cand + j]) ? 0.0 : p; /* filtered block: taken as zero */
                const double G = gi * (pf - (j == pos ? 1.0 : 0.0));
                if (dH)
                    for (int t = 0; t < d; ++t)
                        dh[t] += G * load_elem(E, in_dtype, cand[j] * (int64_t)d + t);
                if (dE) {
                    int64_t row = cand[j];
                    if (row_slot) {
                        row = row_slot[cand[j]];
                        if (row < 0) {
#pragma omp atomic write
                            status = 3;
                            continue;
                        }
                    }
                    for (int t = 0; t < d; ++t) {
                        const double add = G * h[t];
#pragma omp atomic update
                        dE[row * (int64_t)d + t] += add;
                    }
                }
            }
            if (dH)
                for (int t = 0; t < d; ++t)
                    dH[r * d + t] = dh[t];
        }
        free(o);
        free(h);
        free(dh);
        free(cand);
        free(live);
    }
    return status;
}

/*
 * Gradient filtering, block reading (see the header): p is the [n_rows, n_cand]
 * softmax of the VALID positions in batch order.  keep[r, j] = 1 iff the block
 * (r / block, j / block) holds at least one probability >= eps.
 * Returns 0, or 1 for a bad argument.
 */
int cce_oracle_filter_blocks(int64_t n_rows, int64_t n_cand, int32_t block, double eps, const double *p, uint8_t *keep)
{
    if (n_rows < 0 || n_cand <= 0 || block <= 0 || !p || !keep)
        return 1;
    for (int64_t r0 = 0; r0 < n_rows; r0 += block)
        for (int64_t j0 = 0; j0 < n_cand; j0 += block) {
            const int64_t r1 = r0 + block < n_rows ? r0 + block : n_rows;
            const int64_t j1 = j0 + block < n_cand ? j0 + block : n_cand;
            double big = 0.0;
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t j = j0; j < j1; ++j)
                    if (p[r * n_cand + j] > big)
                        big = p[r * n_cand + j];
            const uint8_t k = (big >= eps) ? 1 : 0;
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t j = j0; j < j1; ++j)
                    keep[r * n_cand + j] = k;
        }
    return 0;
}
