/* Driver for a build of oracle/ssa_oracle.c under -fsanitize=address,undefined: every entry point on
 * small inputs that reach its edges (a value tensor that aliases the keys, grouped heads, a ragged
 * row list, the block pattern, several threads, saturating pattern sizes). The sanitizers abort on
 * any out-of-bounds access or undefined arithmetic; the printed sums are compared by
 * tests/test_sanitizers.py with what the ordinary build returns through the Python loader. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_ssa_rows(const void *, const void *, const void *, int, int64_t, const int64_t *, const int64_t *, const int64_t *,
                    int, int, int, int64_t, int, int, int64_t, int64_t, int64_t, int64_t, double, double *, double *, double *, int);
int oracle_ssa_rows_blocks(const void *, const void *, const void *, int, int64_t, const int64_t *, const int64_t *, const int64_t *,
                           int, int, int, int64_t, int, int, int64_t, int64_t, int64_t, int64_t, int64_t, double, double *, double *,
                           double *, int);
int oracle_ssa_live_mask(int64_t, int64_t, int64_t, int64_t, uint8_t *);
int64_t oracle_ssa_count_pairs(int64_t, int64_t, int64_t);
int oracle_ssa_live_mask_blocks(int64_t, int64_t, int64_t, int64_t, int64_t, uint8_t *);
int64_t oracle_ssa_count_pairs_blocks(int64_t, int64_t, int64_t, int64_t);
int oracle_ssa_backward(const void *, const void *, const void *, const void *, int, int, int, int, int64_t, int, int, int64_t,
                        int64_t, int64_t, int64_t, int64_t, double, const void *, const float *, double *, double *, double *, int);
int oracle_ssa_backward_rows(const void *, const void *, const void *, const void *, int, int64_t, const int64_t *,
                             const int64_t *, const int64_t *, int, int, int, int64_t, int, int, int64_t, int64_t, int64_t,
                             int64_t, int64_t, double, const void *, const float *, double *, double *, double *, int);

static uint32_t rng_state = 12345u;
static float rnd(void)
{   /* xorshift, mapped to (-2, 2) in steps that fp32 and bf16 hold exactly */
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 17; rng_state ^= rng_state << 5;
    return (float)((int)(rng_state % 65u) - 32) / 16.0f;
}
static double sum(const double *x, int64_t n) { double s = 0; for (int64_t i = 0; i < n; ++i) s += x[i]; return s; }

int main(void)
{
    enum { B = 2, Hq = 4, Hkv = 2, S = 37, DQK = 12, DV = 8 };
    float *q = malloc(sizeof(float) * B * S * Hq * DQK), *k = malloc(sizeof(float) * B * S * Hkv * DQK);
    float *dout = malloc(sizeof(float) * B * S * Hq * DV);
    for (int i = 0; i < B * S * Hq * DQK; ++i) q[i] = rnd();
    for (int i = 0; i < B * S * Hkv * DQK; ++i) k[i] = rnd();
    for (int i = 0; i < B * S * Hq * DV; ++i) dout[i] = rnd();
    /* rows: all of them, as (b, h, i) lists, queries gathered row by row */
    const int64_t n = (int64_t)B * Hq * S;
    int64_t *rb = malloc(sizeof(int64_t) * n), *rh = malloc(sizeof(int64_t) * n), *ri = malloc(sizeof(int64_t) * n);
    float *q_rows = malloc(sizeof(float) * n * DQK), *dout_rows = malloc(sizeof(float) * n * DV);
    int64_t r = 0;
    for (int b = 0; b < B; ++b) for (int h = 0; h < Hq; ++h) for (int i = 0; i < S; ++i, ++r) {
        rb[r] = b; rh[r] = h; ri[r] = i;
        for (int c = 0; c < DQK; ++c) q_rows[r * DQK + c] = q[((b * S + i) * Hq + h) * DQK + c];
        for (int c = 0; c < DV; ++c) dout_rows[r * DV + c] = dout[((b * S + i) * Hq + h) * DV + c];
    }
    double *out = malloc(sizeof(double) * n * DV), *lse = malloc(sizeof(double) * n), *w = malloc(sizeof(double) * n * S);
    /* values alias the keys (row stride DQK), token pattern, 3 threads, weights requested */
    int rc = oracle_ssa_rows(q_rows, k, k, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 3, 5, 0.25, out, lse, w, 3);
    printf("rows %d %.12e %.12e %.12e\n", rc, sum(out, n * DV), sum(lse, n), sum(w, n * S));
    rc = oracle_ssa_rows(q_rows, k, k, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, INT64_MAX, INT64_MAX, 0.25, out, lse, NULL, 1);
    printf("rows_inf %d %.12e %.12e\n", rc, sum(out, n * DV), sum(lse, n));
    rc = oracle_ssa_rows_blocks(q_rows, k, k, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 1, 2, 4, 0.25, out, lse, w, 2);
    printf("rows_blocks %d %.12e %.12e\n", rc, sum(out, n * DV), sum(lse, n));
    rc = oracle_ssa_rows_blocks(q_rows, k, k, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, INT64_MAX, INT64_MAX, INT64_MAX, 0.25,
                                out, lse, NULL, 2);
    printf("rows_blocks_inf %d %.12e\n", rc, sum(out, n * DV));
    uint8_t mask[S];
    int64_t live = 0;
    for (int i = 0; i < S; ++i) { oracle_ssa_live_mask(i, S, 3, 5, mask); for (int j = 0; j < S; ++j) live += mask[j]; }
    printf("pairs %lld %lld %lld\n", (long long)live, (long long)oracle_ssa_count_pairs(S, 3, 5),
           (long long)oracle_ssa_count_pairs(S, INT64_MAX, INT64_MAX));
    live = 0;
    for (int i = 0; i < S; ++i) { oracle_ssa_live_mask_blocks(i, S, 1, 2, 4, mask); for (int j = 0; j < S; ++j) live += mask[j]; }
    printf("pairs_blocks %lld %lld %lld\n", (long long)live, (long long)oracle_ssa_count_pairs_blocks(S, 1, 2, 4),
           (long long)oracle_ssa_count_pairs_blocks(S, INT64_MAX, INT64_MAX, INT64_MAX));
    /* gradients: dense, then the listed-rows form on the same rows */
    double *dq = malloc(sizeof(double) * n * DQK), *dk = malloc(sizeof(double) * B * S * Hkv * DQK), *dv = malloc(sizeof(double) * B * S * Hkv * DV);
    rc = oracle_ssa_backward(q, k, k, dout, 0, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 3, 5, 0, 0.25, NULL, NULL, dq, dk, dv, 3);
    printf("backward %d %.12e %.12e %.12e\n", rc, sum(dq, n * DQK), sum(dk, (int64_t)B * S * Hkv * DQK), sum(dv, (int64_t)B * S * Hkv * DV));
    rc = oracle_ssa_backward(q, k, k, dout, 0, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 1, 2, 4, 0.25, NULL, NULL, dq, dk, dv, 2);
    printf("backward_blocks %d %.12e %.12e %.12e\n", rc, sum(dq, n * DQK), sum(dk, (int64_t)B * S * Hkv * DQK), sum(dv, (int64_t)B * S * Hkv * DV));
    rc = oracle_ssa_backward_rows(q_rows, k, k, dout_rows, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 3, 5, 0, 0.25, NULL, NULL,
                                  dq, dk, dv, 3);
    printf("backward_rows %d %.12e %.12e %.12e\n", rc, sum(dq, n * DQK), sum(dk, (int64_t)B * S * Hkv * DQK), sum(dv, (int64_t)B * S * Hkv * DV));
    /* rejected arguments return before touching anything */
    printf("bad %d %d %d\n", oracle_ssa_rows(NULL, k, k, 0, n, rb, rh, ri, B, Hq, Hkv, S, DQK, DV, DQK, DQK, 3, 5, 0.25, out, lse, NULL, 1),
           oracle_ssa_rows(q_rows, k, k, 0, n, rb, rh, ri, B, Hq, 3, S, DQK, DV, DQK, DQK, 3, 5, 0.25, out, lse, NULL, 1),
           oracle_ssa_live_mask(S, S, 3, 5, mask));
    free(q); free(k); free(dout); free(rb); free(rh); free(ri); free(q_rows); free(dout_rows);
    free(out); free(lse); free(w); free(dq); free(dk); free(dv);
    return 0;
}
