/*
 * ssa_oracle.c — TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, fp64 CPU definition of streaming sparse attention (SSA), written out from the
 * paper's statement O* = softmax(Q K*) V* (Architecture section, Eq. 2 and Eq. 4): every query
 * attends to a fixed set of leading "sink" keys plus a causal window of recent keys, and the
 * softmax is taken over that restricted key set only.  The pieces the paper leaves implicit
 * (transpose on K, the 1/sqrt(d) scale passed in as `scale`, the normalising denominator, the
 * causal order of a language model) are written in their textbook form.
 *
 * There is no tiling, no online softmax, no range arithmetic and no fusion here: one explicit
 * alive(i, j) predicate per (query, key) pair, a max, a sum of exponentials, a weighted sum.
 * The file shares nothing with the GPU library: no header, no table, no helper.
 *
 * Only tests/, the smoke check and the CPU-baseline leg of the benchmark may call this.
 *
 * Pins (tests/test_oracle_pins.py): hand-enumerated live sets, the paper's own block arithmetic
 * (1 sink block + 7 local blocks of 128 = 1,024 live tokens, Training section), reduction to
 * textbook causal attention for window >= S (Eq. 2 -> Eq. 1) checked against an independent
 * library routine, closed forms for Q = 0 / constant V / single-key rows, shift invariance of
 * the scores, grouped-head mapping, and brute-force masks built from Python sets.  The
 * block-granular pattern is pinned by the paper's printed sizes (block 128, 1 sink block, 7 local
 * blocks: at most 1,024 live tokens), hand-enumerated live sets, its block = 1 case (which is the
 * token-granular pattern) and the same library routine under a mask built from Python sets.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_DTYPE_F32 0
#define ORACLE_DTYPE_BF16 1

/* The sparsity pattern of Eq. 4 at token granularity: key j is visible to query i when it is
 * not in the future (j <= i) and is either one of the first n_sink keys or one of the `window`
 * most recent keys, the query's own position included. */
static int alive(int64_t i, int64_t j, int64_t n_sink, int64_t window)
{
    if (j > i) return 0;
    if (j < n_sink) return 1;
    /* j > i - window, written without overflow for window up to INT64_MAX */
    if (i - j < window) return 1;
    return 0;
}

/* The same pattern as the paper parametrises it (Architecture section, after Eq. 4; values in the
 * Training section): keys and queries are cut into blocks of `block` tokens, and the query in
 * block floor(i / block) sees the first `sink_blocks` key blocks and the `local_blocks` most recent
 * key blocks, its own block counted and cut at the query itself (causal).  With block = 1 this is
 * alive() with n_sink = sink_blocks and window = local_blocks. */
static int alive_blocks(int64_t i, int64_t j, int64_t sink_blocks, int64_t local_blocks, int64_t block)
{
    if (j > i) return 0;
    const int64_t qb = i / block, kb = j / block;
    if (kb < sink_blocks) return 1;
    if (qb - kb < local_blocks) return 1;
    return 0;
}

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_DTYPE_F32) return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

typedef struct {
    const void *q_rows, *k, *v;
    int dtype;
    int64_t n_rows;
    const int64_t *row_b, *row_h, *row_i;
    int Hq, Hkv;
    int64_t S;
    int d_qk, d_v;
    int64_t k_row_stride, v_row_stride; /* elements between consecutive (position, kv-head) rows */
    int64_t n_sink, window; /* tokens; or sink blocks and local blocks when block > 0 */
    int64_t block;          /* 0: token-granular pattern; > 0: block-granular with this block size */
    double scale;
    double *out, *lse, *weights;
    int64_t next_row; /* shared work counter */
    int failed;
} job_t;

/* One query row, straight from the definition. */
static int one_row(job_t *J, int64_t r, double *score /* S doubles */)
{
    const int64_t b = J->row_b[r], h = J->row_h[r], i = J->row_i[r];
    const int group = J->Hq / J->Hkv;
    const int64_t g = h / group; /* query head h reads key/value head g */
    const int64_t S = J->S;
    int64_t n_alive = 0;
    double m = -INFINITY;

    for (int64_t j = 0; j < S; ++j) {
        const int live = J->block > 0 ? alive_blocks(i, j, J->n_sink, J->window, J->block)
                                      : alive(i, j, J->n_sink, J->window);
        if (!live) { score[j] = -INFINITY; continue; }
        const int64_t kbase = ((b * S + j) * J->Hkv + g) * J->k_row_stride;
        double dot = 0.0;
        for (int c = 0; c < J->d_qk; ++c)
            dot += widen(J->q_rows, J->dtype, r * (int64_t)J->d_qk + c) * widen(J->k, J->dtype, kbase + c);
        score[j] = J->scale * dot;
        if (score[j] > m) m = score[j];
        ++n_alive;
    }
    if (n_alive == 0) return -1; /* softmax over an empty set is undefined */

    double l = 0.0;
    for (int64_t j = 0; j < S; ++j)
        if (score[j] != -INFINITY) l += exp(score[j] - m);

    double *o = J->out + r * (int64_t)J->d_v;
    for (int c = 0; c < J->d_v; ++c) o[c] = 0.0;
    for (int64_t j = 0; j < S; ++j) {
        double w = (score[j] == -INFINITY) ? 0.0 : exp(score[j] - m) / l;
        if (J->weights) J->weights[r * S + j] = w;
        if (w == 0.0 && score[j] == -INFINITY) continue;
        const int64_t vbase = ((b * S + j) * J->Hkv + g) * J->v_row_stride;
        for (int c = 0; c < J->d_v; ++c) o[c] += w * widen(J->v, J->dtype, vbase + c);
    }
    J->lse[r] = m + log(l);
    return 0;
}

static void *worker(void *arg)
{
    job_t *J = (job_t *)arg;
    double *score = (double *)malloc((size_t)J->S * sizeof(double));
    if (!score) { __atomic_store_n(&J->failed, 1, __ATOMIC_SEQ_CST); return NULL; }
    for (;;) {
        int64_t r = __atomic_fetch_add(&J->next_row, 1, __ATOMIC_SEQ_CST);
        if (r >= J->n_rows) break;
        if (one_row(J, r, score) != 0) __atomic_store_n(&J->failed, 2, __ATOMIC_SEQ_CST);
    }
    free(score);
    return NULL;
}

/*
 * SSA for a list of query rows (Eq. 4; Eq. 1 when window >= S).
 *
 *   q_rows   [n_rows, d_qk]            the query vectors of the listed rows, gathered
 *   k        [B, S, Hkv, k_row_stride] keys   (first d_qk elements of each row are used)
 *   v        [B, S, Hkv, v_row_stride] values (first d_v elements of each row are used);
 *                                      v may alias k (absorbed MLA: V is a prefix of the latent)
 *   row_b/h/i[n_rows]                  batch index, query head, query position of each row
 *   out      [n_rows, d_v] fp64, lse [n_rows] fp64 (natural log of the softmax denominator)
 *   weights  NULL or [n_rows, S] fp64: the attention weights themselves (0 exactly where dead)
 *
 * A decode step is the row i = L - 1 of a cache whose rows j >= L are never alive (j > i).
 * Returns 0, or -1 on a bad argument, -2 if a row has no live key, -3 on allocation failure.
 */
static int run_rows(const void *q_rows, const void *k, const void *v, int dtype,
                    int64_t n_rows, const int64_t *row_b, const int64_t *row_h, const int64_t *row_i,
                    int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                    int64_t k_row_stride, int64_t v_row_stride,
                    int64_t n_sink, int64_t window, int64_t block, double scale,
                    double *out, double *lse, double *weights, int n_threads)
{
    if (!q_rows || !k || !v || !out || !lse) return -1;
    if (dtype != ORACLE_DTYPE_F32 && dtype != ORACLE_DTYPE_BF16) return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || d_qk < 1 || d_v < 1) return -1;
    if (k_row_stride < d_qk || v_row_stride < d_v || n_sink < 0 || window < 1) return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (row_b[r] < 0 || row_b[r] >= B || row_h[r] < 0 || row_h[r] >= Hq || row_i[r] < 0 || row_i[r] >= S)
            return -1;

    job_t J;
    memset(&J, 0, sizeof J);
    J.q_rows = q_rows; J.k = k; J.v = v; J.dtype = dtype; J.n_rows = n_rows;
    J.row_b = row_b; J.row_h = row_h; J.row_i = row_i; J.Hq = Hq; J.Hkv = Hkv; J.S = S;
    J.d_qk = d_qk; J.d_v = d_v; J.k_row_stride = k_row_stride; J.v_row_stride = v_row_stride;
    J.n_sink = n_sink; J.window = window; J.block = block; J.scale = scale;
    J.out = out; J.lse = lse; J.weights = weights;

    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    if ((int64_t)n_threads > n_rows) n_threads = (int)(n_rows > 0 ? n_rows : 1);
    pthread_t tid[256];
    int started = 0;
    for (int t = 1; t < n_threads; ++t)
        if (pthread_create(&tid[started], NULL, worker, &J) == 0) ++started;
    worker(&J);
    for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
    if (J.failed == 1) return -3;
    if (J.failed == 2) return -2;
    return 0;
}

int oracle_ssa_rows(const void *q_rows, const void *k, const void *v, int dtype,
                    int64_t n_rows, const int64_t *row_b, const int64_t *row_h, const int64_t *row_i,
                    int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                    int64_t k_row_stride, int64_t v_row_stride,
                    int64_t n_sink, int64_t window, double scale,
                    double *out, double *lse, double *weights, int n_threads)
{
    return run_rows(q_rows, k, v, dtype, n_rows, row_b, row_h, row_i, B, Hq, Hkv, S, d_qk, d_v,
                    k_row_stride, v_row_stride, n_sink, window, 0, scale, out, lse, weights, n_threads);
}

/* The same for the block-granular pattern: `sink_blocks` >= 0, `local_blocks` >= 1, `block` >= 1. */
int oracle_ssa_rows_blocks(const void *q_rows, const void *k, const void *v, int dtype,
                           int64_t n_rows, const int64_t *row_b, const int64_t *row_h, const int64_t *row_i,
                           int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                           int64_t k_row_stride, int64_t v_row_stride,
                           int64_t sink_blocks, int64_t local_blocks, int64_t block, double scale,
                           double *out, double *lse, double *weights, int n_threads)
{
    if (block < 1) return -1;
    return run_rows(q_rows, k, v, dtype, n_rows, row_b, row_h, row_i, B, Hq, Hkv, S, d_qk, d_v,
                    k_row_stride, v_row_stride, sink_blocks, local_blocks, block, scale, out, lse, weights,
                    n_threads);
}

/* The live set of one query as an explicit 0/1 vector over keys 0..S-1 (Eq. 4's pattern). */
int oracle_ssa_live_mask(int64_t i, int64_t S, int64_t n_sink, int64_t window, uint8_t *mask)
{
    if (!mask || S < 1 || i < 0 || i >= S || n_sink < 0 || window < 1) return -1;
    for (int64_t j = 0; j < S; ++j) mask[j] = (uint8_t)alive(i, j, n_sink, window);
    return 0;
}

/* Number of live (query, key) pairs of a causal length-S prefill, by counting them one by one. */
int64_t oracle_ssa_count_pairs(int64_t S, int64_t n_sink, int64_t window)
{
    int64_t n = 0;
    for (int64_t i = 0; i < S; ++i)
        for (int64_t j = 0; j <= i; ++j) n += alive(i, j, n_sink, window);
    return n;
}

/* The block-granular live set of one query as a 0/1 vector over keys 0..S-1. */
int oracle_ssa_live_mask_blocks(int64_t i, int64_t S, int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                uint8_t *mask)
{
    if (!mask || S < 1 || i < 0 || i >= S || sink_blocks < 0 || local_blocks < 1 || block < 1) return -1;
    for (int64_t j = 0; j < S; ++j) mask[j] = (uint8_t)alive_blocks(i, j, sink_blocks, local_blocks, block);
    return 0;
}

/* Live (query, key) pairs of a causal length-S prefill under the block-granular pattern, one by one. */
int64_t oracle_ssa_count_pairs_blocks(int64_t S, int64_t sink_blocks, int64_t local_blocks, int64_t block)
{
    int64_t n = 0;
    for (int64_t i = 0; i < S; ++i)
        for (int64_t j = 0; j <= i; ++j) n += alive_blocks(i, j, sink_blocks, local_blocks, block);
    return n;
}

/* ------------------------------------------------------------------------------------------------
 * Gradient of SSA (what the sparse mid-training of the Architecture section's Training paragraph
 * differentiates): for the scalar L = sum over rows of <dO_row, O_row>, with O from Eq. 4 under the
 * same live sets, the derivatives with respect to Q, K and V by the chain rule of a softmax:
 *
 *   p_ij  = exp(scale q_i.k_j - lse_i)   for live j, 0 otherwise
 *   dV_j  = sum_i p_ij dO_i
 *   dP_ij = dO_i . v_j ,   D_i = dO_i . O_i (= sum_j p_ij dP_ij)
 *   dS_ij = p_ij (dP_ij - D_i)
 *   dQ_i  = scale sum_j dS_ij k_j ,   dK_j = scale sum_i dS_ij q_i
 *
 * (sums over i run over every query row -- all heads of the key's group -- that sees key j).
 * By default nothing is saved from a forward pass: every row's scores, maximum, denominator and
 * output are recomputed here from the definition.  A training step does not recompute them: it
 * hands the backward the `out` and `lse` its forward produced, rounded to their storage types, and
 * takes D_i and p_ij from those.  With `out_saved` / `lse_saved` given, this file does the same
 * substitution (D_i = dO_i . out_saved_i, p_ij = exp(scale q_i.k_j - lse_saved_i)) and nothing else
 * changes; given its own forward's values it returns the gradient itself.  A row whose dO is zero
 * everywhere contributes exactly nothing and is skipped, which lets a test at full sequence length
 * put its dO on a few rows.
 * dK and dV are always returned separately; when V is a prefix of K (absorbed MLA) the gradient
 * with respect to the shared tensor is their sum, which the caller forms.
 *
 * Pins (tests/test_oracle_pins_backward.py): reverse-mode differentiation of a library attention
 * routine under a mask built from Python sets, central finite differences of this file's own
 * forward, the closed form for Q = 0, and the row-sum identities sum_j dS_ij = 0.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    const void *q, *k, *v, *dout;
    const void *out_saved;   /* NULL, or [B, S, Hq, d_v] in the inputs' dtype */
    const float *lse_saved;  /* NULL, or [B, Hq, S] fp32 */
    int dtype;
    int B, Hq, Hkv;
    int64_t S;
    int d_qk, d_v;
    int64_t k_row_stride, v_row_stride;
    int64_t n_sink, window, block;
    double scale;
    int64_t n_rows;
    const int64_t *rows;   /* flat (b * S + i) * Hq + h of the rows with a nonzero dO */
    int compact;           /* q, dout, out_saved, lse_saved, dq hold the listed rows only, in list order */
    double *row_lse, *row_D;
    double *dq, *dk, *dv;
    int64_t next;          /* shared work counter */
    int failed;
} bwd_t;

static int bwd_alive(const bwd_t *J, int64_t i, int64_t j)
{
    return J->block > 0 ? alive_blocks(i, j, J->n_sink, J->window, J->block) : alive(i, j, J->n_sink, J->window);
}

/* pass 1, one row: forward from the definition, then dQ of the row; keeps lse and D of the row */
static int bwd_row(bwd_t *J, int64_t r, double *score, double *o)
{
    const int64_t flat = J->rows[r];
    const int64_t h = flat % J->Hq, bi = flat / J->Hq, i = bi % J->S, b = bi / J->S;
    const int64_t g = h / (J->Hq / J->Hkv);
    const int64_t S = J->S;
    const int64_t at = J->compact ? r : flat;   /* where this row sits in q, dout, out_saved, dq */
    const int64_t qbase = at * J->d_qk, dobase = at * J->d_v;
    double m = -INFINITY;
    int64_t n_alive = 0;
    for (int64_t j = 0; j < S; ++j) {
        if (!bwd_alive(J, i, j)) { score[j] = -INFINITY; continue; }
        const int64_t kbase = ((b * S + j) * J->Hkv + g) * J->k_row_stride;
        double dot = 0.0;
        for (int c = 0; c < J->d_qk; ++c) dot += widen(J->q, J->dtype, qbase + c) * widen(J->k, J->dtype, kbase + c);
        score[j] = J->scale * dot;
        if (score[j] > m) m = score[j];
        ++n_alive;
    }
    if (n_alive == 0) return -1;
    double l = 0.0;
    for (int64_t j = 0; j < S; ++j)
        if (score[j] != -INFINITY) l += exp(score[j] - m);
    double lse = m + log(l);
    if (J->lse_saved) lse = (double)J->lse_saved[J->compact ? r : (b * J->Hq + h) * S + i];
    if (J->out_saved) {
        for (int c = 0; c < J->d_v; ++c) o[c] = widen(J->out_saved, J->dtype, dobase + c);
    } else {
        for (int c = 0; c < J->d_v; ++c) o[c] = 0.0;
        for (int64_t j = 0; j < S; ++j) {
            if (score[j] == -INFINITY) continue;
            const double p = exp(score[j] - lse);
            const int64_t vbase = ((b * S + j) * J->Hkv + g) * J->v_row_stride;
            for (int c = 0; c < J->d_v; ++c) o[c] += p * widen(J->v, J->dtype, vbase + c);
        }
    }
    double D = 0.0;
    for (int c = 0; c < J->d_v; ++c) D += widen(J->dout, J->dtype, dobase + c) * o[c];
    double *dq = J->dq + qbase;
    for (int c = 0; c < J->d_qk; ++c) dq[c] = 0.0;
    for (int64_t j = 0; j < S; ++j) {
        if (score[j] == -INFINITY) continue;
        const double p = exp(score[j] - lse);
        const int64_t vbase = ((b * S + j) * J->Hkv + g) * J->v_row_stride;
        const int64_t kbase = ((b * S + j) * J->Hkv + g) * J->k_row_stride;
        double dP = 0.0;
        for (int c = 0; c < J->d_v; ++c) dP += widen(J->dout, J->dtype, dobase + c) * widen(J->v, J->dtype, vbase + c);
        const double dS = p * (dP - D);
        for (int c = 0; c < J->d_qk; ++c) dq[c] += J->scale * dS * widen(J->k, J->dtype, kbase + c);
    }
    J->row_lse[r] = lse;
    J->row_D[r] = D;
    return 0;
}

static void *bwd_worker_rows(void *arg)
{
    bwd_t *J = (bwd_t *)arg;
    double *score = (double *)malloc((size_t)J->S * sizeof(double));
    double *o = (double *)malloc((size_t)J->d_v * sizeof(double));
    if (!score || !o) { __atomic_store_n(&J->failed, 1, __ATOMIC_SEQ_CST); free(score); free(o); return NULL; }
    for (;;) {
        int64_t r = __atomic_fetch_add(&J->next, 1, __ATOMIC_SEQ_CST);
        if (r >= J->n_rows) break;
        if (bwd_row(J, r, score, o) != 0) __atomic_store_n(&J->failed, 2, __ATOMIC_SEQ_CST);
    }
    free(score); free(o);
    return NULL;
}

/* pass 2, one key (b, j, g): dK and dV of that key, summed over the rows that see it in list order */
static void bwd_key(bwd_t *J, int64_t key)
{
    const int64_t g = key % J->Hkv, bj = key / J->Hkv, j = bj % J->S, b = bj / J->S;
    const int group = J->Hq / J->Hkv;
    const int64_t kbase = key * J->k_row_stride, vbase = key * J->v_row_stride;
    double *dk = J->dk + key * (int64_t)J->d_qk, *dv = J->dv + key * (int64_t)J->d_v;
    for (int64_t r = 0; r < J->n_rows; ++r) {
        const int64_t flat = J->rows[r];
        const int64_t h = flat % J->Hq, bi = flat / J->Hq, i = bi % J->S, rb = bi / J->S;
        if (rb != b || h / group != g || !bwd_alive(J, i, j)) continue;
        const int64_t at = J->compact ? r : flat;
        const int64_t qbase = at * J->d_qk, dobase = at * J->d_v;
        double dot = 0.0, dP = 0.0;
        for (int c = 0; c < J->d_qk; ++c) dot += widen(J->q, J->dtype, qbase + c) * widen(J->k, J->dtype, kbase + c);
        for (int c = 0; c < J->d_v; ++c) dP += widen(J->dout, J->dtype, dobase + c) * widen(J->v, J->dtype, vbase + c);
        const double p = exp(J->scale * dot - J->row_lse[r]);
        const double dS = p * (dP - J->row_D[r]);
        for (int c = 0; c < J->d_qk; ++c) dk[c] += J->scale * dS * widen(J->q, J->dtype, qbase + c);
        for (int c = 0; c < J->d_v; ++c) dv[c] += p * widen(J->dout, J->dtype, dobase + c);
    }
}

static void *bwd_worker_keys(void *arg)
{
    bwd_t *J = (bwd_t *)arg;
    const int64_t n_keys = (int64_t)J->B * J->S * J->Hkv;
    for (;;) {
        int64_t key = __atomic_fetch_add(&J->next, 1, __ATOMIC_SEQ_CST);
        if (key >= n_keys) break;
        bwd_key(J, key);
    }
    return NULL;
}

static void bwd_run(bwd_t *J, void *(*fn)(void *), int n_threads)
{
    pthread_t tid[256];
    int started = 0;
    J->next = 0;
    for (int t = 1; t < n_threads; ++t)
        if (pthread_create(&tid[started], NULL, fn, J) == 0) ++started;
    fn(J);
    for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
}

/*
 *   q    [B, S, Hq, d_qk]            dout [B, S, Hq, d_v]
 *   k    [B, S, Hkv, k_row_stride]   v    [B, S, Hkv, v_row_stride]  (v may alias k, as in the forward)
 *   dq   [B, S, Hq, d_qk] fp64       dk   [B, S, Hkv, d_qk] fp64       dv [B, S, Hkv, d_v] fp64
 *   block = 0: token-granular pattern (n_sink, window in tokens); block > 0: sink blocks, local blocks.
 *   out_saved, lse_saved: both NULL (recompute the forward), or what a forward pass stored.
 * Returns 0, -1 on a bad argument, -2 if a contributing row has no live key, -3 on allocation failure.
 */
int oracle_ssa_backward(const void *q, const void *k, const void *v, const void *dout, int dtype,
                        int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                        int64_t k_row_stride, int64_t v_row_stride,
                        int64_t n_sink, int64_t window, int64_t block, double scale,
                        const void *out_saved, const float *lse_saved,
                        double *dq, double *dk, double *dv, int n_threads)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv) return -1;
    if ((out_saved == NULL) != (lse_saved == NULL)) return -1;
    if (dtype != ORACLE_DTYPE_F32 && dtype != ORACLE_DTYPE_BF16) return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || d_qk < 1 || d_v < 1) return -1;
    if (k_row_stride < d_qk || v_row_stride < d_v || n_sink < 0 || window < 1 || block < 0) return -1;

    const int64_t n_all = (int64_t)B * S * Hq;
    int64_t *rows = (int64_t *)malloc((size_t)n_all * sizeof(int64_t));
    if (!rows) return -3;
    int64_t n_rows = 0;
    for (int64_t r = 0; r < n_all; ++r) {
        int any = 0;
        for (int c = 0; c < d_v && !any; ++c) any = widen(dout, dtype, r * d_v + c) != 0.0;
        if (any) rows[n_rows++] = r;
    }
    memset(dq, 0, (size_t)n_all * d_qk * sizeof(double));
    memset(dk, 0, (size_t)B * S * Hkv * d_qk * sizeof(double));
    memset(dv, 0, (size_t)B * S * Hkv * d_v * sizeof(double));

    bwd_t J;
    memset(&J, 0, sizeof J);
    J.q = q; J.k = k; J.v = v; J.dout = dout; J.dtype = dtype; J.B = B; J.Hq = Hq; J.Hkv = Hkv; J.S = S;
    J.d_qk = d_qk; J.d_v = d_v; J.k_row_stride = k_row_stride; J.v_row_stride = v_row_stride;
    J.n_sink = n_sink; J.window = window; J.block = block; J.scale = scale;
    J.n_rows = n_rows; J.rows = rows; J.dq = dq; J.dk = dk; J.dv = dv;
    J.out_saved = out_saved; J.lse_saved = lse_saved;
    J.row_lse = (double *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(double));
    J.row_D = (double *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(double));
    if (!J.row_lse || !J.row_D) { free(rows); free(J.row_lse); free(J.row_D); return -3; }
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    bwd_run(&J, bwd_worker_rows, n_threads);
    if (!J.failed) bwd_run(&J, bwd_worker_keys, n_threads);
    free(rows); free(J.row_lse); free(J.row_D);
    if (J.failed == 1) return -3;
    if (J.failed == 2) return -2;
    return 0;
}

/*
 * The same for a list of query rows given on their own (every other row taken to have dO = 0):
 *   q_rows [n, d_qk], dout_rows [n, d_v], row_b/h/i [n]; out_rows [n, d_v] and lse_rows [n] (fp32) as
 *   out_saved / lse_saved above, or both NULL; dq_rows [n, d_qk] fp64; dk, dv dense as above.
 * This is what lets a test at full sequence length check every dK and dV row: the device computes
 * with a dense dO that is zero outside the listed rows.
 */
int oracle_ssa_backward_rows(const void *q_rows, const void *k, const void *v, const void *dout_rows, int dtype,
                             int64_t n_rows, const int64_t *row_b, const int64_t *row_h, const int64_t *row_i,
                             int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                             int64_t k_row_stride, int64_t v_row_stride,
                             int64_t n_sink, int64_t window, int64_t block, double scale,
                             const void *out_rows, const float *lse_rows,
                             double *dq_rows, double *dk, double *dv, int n_threads)
{
    if (!q_rows || !k || !v || !dout_rows || !dq_rows || !dk || !dv || n_rows < 0) return -1;
    if ((out_rows == NULL) != (lse_rows == NULL)) return -1;
    if (dtype != ORACLE_DTYPE_F32 && dtype != ORACLE_DTYPE_BF16) return -1;
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || S < 1 || d_qk < 1 || d_v < 1) return -1;
    if (k_row_stride < d_qk || v_row_stride < d_v || n_sink < 0 || window < 1 || block < 0) return -1;
    int64_t *rows = (int64_t *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int64_t));
    if (!rows) return -3;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (row_b[r] < 0 || row_b[r] >= B || row_h[r] < 0 || row_h[r] >= Hq || row_i[r] < 0 || row_i[r] >= S) {
            free(rows);
            return -1;
        }
        rows[r] = (row_b[r] * S + row_i[r]) * Hq + row_h[r];
    }
    memset(dk, 0, (size_t)B * S * Hkv * d_qk * sizeof(double));
    memset(dv, 0, (size_t)B * S * Hkv * d_v * sizeof(double));
    bwd_t J;
    memset(&J, 0, sizeof J);
    J.q = q_rows; J.k = k; J.v = v; J.dout = dout_rows; J.dtype = dtype; J.B = B; J.Hq = Hq; J.Hkv = Hkv; J.S = S;
    J.d_qk = d_qk; J.d_v = d_v; J.k_row_stride = k_row_stride; J.v_row_stride = v_row_stride;
    J.n_sink = n_sink; J.window = window; J.block = block; J.scale = scale;
    J.n_rows = n_rows; J.rows = rows; J.compact = 1; J.dq = dq_rows; J.dk = dk; J.dv = dv;
    J.out_saved = out_rows; J.lse_saved = lse_rows;
    J.row_lse = (double *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(double));
    J.row_D = (double *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(double));
    if (!J.row_lse || !J.row_D) { free(rows); free(J.row_lse); free(J.row_D); return -3; }
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    bwd_run(&J, bwd_worker_rows, n_threads);
    if (!J.failed) bwd_run(&J, bwd_worker_keys, n_threads);
    free(rows); free(J.row_lse); free(J.row_D);
    if (J.failed == 1) return -3;
    if (J.failed == 2) return -2;
    return 0;
}
