/*
 * Sanitizer driver of the CPU oracle (test infrastructure).  Built by tests/test_sanitizers.py together with
 * oracle/cce_oracle.c under -fsanitize=address,undefined and run as a program of its own: small cases of every mode,
 * dtype and optional argument, including the error returns, so that an out-of-bounds read or write, a misaligned or
 * overflowing index computation or a leak in the checker itself is found by the compiler's run-time checks.  It
 * prints nothing but a final "ok"; results are not judged here (the pins do that).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int cce_oracle_run(int64_t N, int64_t V, int32_t d, int32_t K, int32_t in_dtype, int32_t neg_mode,
                   int32_t mask_collisions, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                   const uint8_t *mask, const double *g, int64_t n_sel, const int64_t *sel, double *loss, double *lse,
                   double *dH, const int64_t *row_slot, double *dE, double *p_out, const uint8_t *p_keep);
int cce_oracle_filter_blocks(int64_t n_rows, int64_t n_cand, int32_t block, double eps, const double *p, uint8_t *keep);
int cce_oracle_num_threads(void);

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
static float next_unit(void) { return (float)(next_u32() % 2001) / 1000.0f - 1.0f; }

static int run_case(int N, int V, int d, int K, int dtype, int mode, int collide, int with_mask, int with_sel, int compact)
{
    const size_t esz = dtype == 0 ? 4 : 2;
    void *H = malloc((size_t)N * d * esz), *E = malloc((size_t)V * d * esz);
    for (size_t i = 0; i < (size_t)N * d; ++i) {
        float f = next_unit();
        if (dtype == 0) ((float *)H)[i] = f;
        else { uint32_t b; memcpy(&b, &f, 4); ((uint16_t *)H)[i] = (uint16_t)(b >> 16); }
    }
    for (size_t i = 0; i < (size_t)V * d; ++i) {
        float f = 0.3f * next_unit();
        if (dtype == 0) ((float *)E)[i] = f;
        else { uint32_t b; memcpy(&b, &f, 4); ((uint16_t *)E)[i] = (uint16_t)(b >> 16); }
    }
    int32_t *tgt = malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    for (int i = 0; i < N; ++i) tgt[i] = (int32_t)(next_u32() % (uint32_t)V);
    const size_t n_neg = mode == 0 ? (size_t)K : (mode == 1 ? (size_t)N * K : 0);
    int32_t *neg = n_neg ? malloc(sizeof(int32_t) * n_neg) : NULL;
    for (size_t i = 0; i < n_neg; ++i) neg[i] = (int32_t)(next_u32() % (uint32_t)V);
    uint8_t *mask = NULL;
    if (with_mask) {
        mask = malloc((size_t)(N > 0 ? N : 1));
        for (int i = 0; i < N; ++i) mask[i] = (next_u32() % 4) != 0;
    }
    int64_t n_out = N, *sel = NULL;
    if (with_sel) {
        n_out = (N + 1) / 2;
        sel = malloc(sizeof(int64_t) * (size_t)(n_out > 0 ? n_out : 1));
        for (int64_t r = 0; r < n_out; ++r) sel[r] = (2 * r) % (N > 0 ? N : 1);
    }
    const int64_t n_cand = mode == 2 ? V : K + 1;
    double *g = malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    for (int i = 0; i < N; ++i) g[i] = next_unit();
    double *loss = calloc((size_t)(n_out > 0 ? n_out : 1), sizeof(double)), *lse = calloc((size_t)(n_out > 0 ? n_out : 1), sizeof(double));
    double *dH = calloc((size_t)(n_out > 0 ? n_out : 1) * d, sizeof(double));
    double *p = calloc((size_t)(n_out > 0 ? n_out : 1) * n_cand, sizeof(double));
    int64_t *slot = NULL;
    int64_t dE_rows = V;
    if (compact) {  /* every item gets a slot, in reverse order */
        slot = malloc(sizeof(int64_t) * (size_t)V);
        for (int64_t v = 0; v < V; ++v) slot[v] = V - 1 - v;
    }
    double *dE = calloc((size_t)dE_rows * d, sizeof(double));
    int rc = cce_oracle_run(N, V, d, K, dtype, mode, collide, H, E, tgt, neg, mask, g, n_out, sel, loss, lse, dH, slot, dE, p, NULL);
    if (rc == 0 && n_out > 0) {  /* gradient filtering marks on the softmax just produced, applied in a second run */
        uint8_t *keep = malloc((size_t)n_out * n_cand);
        rc = cce_oracle_filter_blocks(n_out, n_cand, 3, 0.05, p, keep);
        if (rc == 0)
            rc = cce_oracle_run(N, V, d, K, dtype, mode, collide, H, E, tgt, neg, mask, NULL, n_out, sel, loss, lse, NULL, slot, dE, NULL, keep);
        free(keep);
    }
    for (int64_t r = 0; r < n_out && rc == 0; ++r)
        if (!isfinite(loss[r]) || !isfinite(lse[r])) rc = 100;
    free(H); free(E); free(tgt); free(neg); free(mask); free(sel); free(g); free(loss); free(lse); free(dH); free(p); free(slot); free(dE);
    return rc;
}

int main(void)
{
    if (cce_oracle_num_threads() < 1) return 2;
    int cases = 0;
    for (int mode = 0; mode < 3; ++mode)
        for (int dtype = 0; dtype < 2; ++dtype)
            for (int variant = 0; variant < 8; ++variant) {
                const int N = (variant == 7) ? 1 : 5 + variant, V = 11 + 3 * variant, d = 1 + 2 * variant;
                const int K = (mode == 2) ? 0 : (variant == 6 ? 0 : 2 + variant);
                const int rc = run_case(N, V, d, K, dtype, mode, variant & 1, (variant >> 1) & 1, (variant >> 2) & 1, variant % 3 == 0);
                if (rc != 0) {
                    fprintf(stderr, "case mode=%d dtype=%d variant=%d returned %d\n", mode, dtype, variant, rc);
                    return 1;
                }
                ++cases;
            }
    /* error returns: bad arguments, an id out of range, a missing compact slot */
    double one[8] = {0}, out[8] = {0};
    float h[4] = {1, 2, 3, 4}, e[8] = {1, 0, 0, 1, 1, 1, 0, 0};
    int32_t tgt[1] = {1}, neg[2] = {0, 5};
    int64_t slot[2] = {0, -1};
    if (cce_oracle_run(1, 2, 4, 2, 0, 0, 1, h, e, tgt, NULL, NULL, NULL, 0, NULL, one, one + 1, NULL, NULL, NULL, NULL, NULL) != 1) return 3;
    if (cce_oracle_run(1, 2, 4, 2, 0, 0, 1, h, e, tgt, neg, NULL, NULL, 0, NULL, one, one + 1, NULL, NULL, NULL, NULL, NULL) != 2) return 4;
    neg[1] = 0;
    if (cce_oracle_run(1, 2, 4, 2, 0, 0, 0, h, e, tgt, neg, NULL, NULL, 0, NULL, one, one + 1, NULL, slot, out, NULL, NULL) != 3) return 5;
    if (cce_oracle_run(0, 2, 4, 0, 0, 2, 0, h, e, tgt, NULL, NULL, NULL, 0, NULL, one, one + 1, NULL, NULL, NULL, NULL, NULL) != 0) return 6;
    printf("ok %d cases\n", cases);
    return 0;
}
