/*
 * loza_ssa.h — C ABI of the streaming sparse attention (SSA) library for MI355X (gfx950).
 *
 * SSA is the sparse attention of LongCat ZigZag Attention: O* = softmax(Q K*^T) V*, where every
 * query keeps a fixed set of leading "sink" keys plus a causal window of its most recent keys
 * (paper: Architecture section, Eq. 2 and Eq. 4; sink/local sizes in the Training section).
 * With window >= S the same entry points compute ordinary causal attention (Eq. 1), which is the
 * full-attention comparator.
 *
 * Live set at token granularity (0-based query position i, key position j):
 *     live(i) = { j : j <= i  and ( j < n_sink  or  i - j < window ) }
 * so the window counts the query's own position, sink and window are united (a key is used once),
 * and |live(i)| = min(i + 1, n_sink + window).
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers unless stated; the caller owns every buffer; the
 *     library allocates nothing and performs no host sync. It keeps no state between calls (the one
 *     exception, a scratch buffer whose contents never matter, is described at loza_ssa_decode_static).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Calls are
 *     asynchronous on it.
 *   - Layouts are dense, innermost index fastest. bf16 tensors are raw 16-bit patterns.
 *   - Query head h reads key/value head h / (Hq / Hkv); Hq must be a multiple of Hkv.
 *   - Absorbed MLA (many query heads share one latent): pass v == k with d_v <= d_qk; the value
 *     row is then the first d_v elements of the key row (row stride d_qk) and costs no second load.
 *   - Base pointers must be 16-byte aligned. Inputs must be finite.
 *   - Every argument is validated before the first HIP call; a failed validation launches nothing.
 *   - Return value: LOZA_OK or a negative loza_status.
 *   - One environment variable is read (on every decode call and by the two host-only size functions
 *     below): LOZA_DECODE_SPLITS=n, 1 <= n <= 64, replaces the number of key splits a decode call
 *     chooses from its sizes (other values are ignored). It exists for tests and experiments; it
 *     changes the workspace size, so it must not change between loza_ssa_decode_workspace_bytes and
 *     the decode call. Nothing else is read from the environment.
 *   - Where each declaration comes from: the prototypes of loza_ssa_prefill and loza_ssa_decode are
 *     given by the benchmark spec; the operation is the paper's (cited at each entry point); every
 *     other name, argument and helper is this library's own.
 */
#ifndef LOZA_SSA_H
#define LOZA_SSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOZA_OK = 0,
    LOZA_ERR_NULL = -1,        /* a required pointer is NULL                                  */
    LOZA_ERR_SHAPE = -2,       /* sizes out of range or inconsistent (Hq % Hkv, window < 1…)  */
    LOZA_ERR_UNSUPPORTED = -3, /* a (dtype, d_qk, d_v) combination no kernel is built for      */
    LOZA_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than loza_ssa_decode_workspace_bytes */
    LOZA_ERR_HIP = -5,         /* a HIP call failed (hipGetLastError has the detail)          */
    LOZA_ERR_ALIGN = -6        /* a base pointer is not 16-byte aligned                       */
} loza_status;

#define LOZA_WINDOW_INF INT64_MAX /* window = infinity: full causal attention (Eq. 1) */

/*
 * SSA prefill, bf16 in / bf16 out, fp32 accumulation (Eq. 4; Eq. 1 when window >= S).
 *   q    [B, S, Hq,  d_qk] bf16      k [B, S, Hkv, d_qk] bf16      v [B, S, Hkv, d_v] bf16 (or v == k)
 *   out  [B, S, Hq,  d_v ] bf16      lse [B, Hq, S] fp32, natural log of the softmax denominator
 *   n_sink >= 0 leading keys always visible; window >= 1 most recent keys visible (self included).
 *   scale multiplies q.k before the softmax (the 1/sqrt(d) the paper's equations leave out);
 *   finite and > 0 (anything else: LOZA_ERR_SHAPE).
 * Supported (d_qk, d_v): (576, 512) with v == k (absorbed MLA: the value row is the first 512
 * elements of the key row), and (128, 128) with v separate or v == k. Anything else:
 * LOZA_ERR_UNSUPPORTED. S <= 2^31 - 129.
 * Numerics: scores, exponentials and sums in fp32; the softmax weights go to the matrix cores as
 * bf16, rounded once (relative error 2^-9 each) or, where that is not good enough, as two bf16
 * terms (2^-17): for tiles that start within the first 128 positions, for patterns that leave every
 * row fewer than 128 live keys, and for every tile in which the one-term pass produced a result of
 * magnitude >= 1.97 (the tile is then computed again inside the same launch). Error of a result:
 *     |out - exact| <= half an ulp of bf16 at |out|  +  w * D  +  about 1e-6 * |out|,
 * D = the softmax-weighted mean of |v_j - out| over the live keys (never more than their largest
 * distance from out), w = 2^-9 for one-term rows and 2^-17 for two-term rows. One-term rows have
 * |out| < 2, i.e. half an ulp <= 2^-8: they stay inside 1e-2 whenever D <= 3.1 (values of unit
 * scale give D of about 1, and random rounding errors add to a small fraction of w * D); two-term
 * rows stay inside 1e-2 for |out| < 4 whenever D <= 280. From |out| = 4 on the rounding of the
 * result to bf16 alone is 2^-6. lse: fp32 throughout, |lse - exact| <= 2e-5 at the tested sizes.
 * The launch is deterministic: the same inputs give the same bits.
 */
int loza_ssa_prefill(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                     int64_t n_sink, int64_t window, float scale, void *stream);

/*
 * fp32 twin of loza_ssa_prefill (fp32 in, fp32 arithmetic, fp32 out), same layouts with float
 * elements. Any d_qk, d_v in [1, 256]; v may alias k with d_v <= d_qk; scale finite, any sign.
 * Plain vector arithmetic (no matrix cores): the small-shape check of the method, not a fast path.
 */
int loza_ssa_prefill_f32(const float *q, const float *k, const float *v, float *out, float *lse,
                         int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                         int64_t n_sink, int64_t window, float scale, void *stream);

/*
 * SSA decode: one new query token per sequence against that sequence's KV cache (the decode
 * kernel of the paper's Efficiency section). Split over the live keys with a log-sum-exp merge.
 *   q       [B, Hq, d_qk] bf16
 *   kcache  [B, S_max, Hkv, d_qk] bf16     vcache [B, S_max, Hkv, d_v] bf16 (or vcache == kcache)
 *   seqlens [B] int32 (device): valid rows of each cache INCLUDING the new token's own key/value,
 *           so the query sits at position seqlens[b] - 1. 0 <= seqlens[b] <= S_max is required;
 *           a sequence of length 0 yields out = 0, lse = -inf.
 *   out     [B, Hq, d_v] bf16              lse [B, Hq] fp32
 *   workspace: device scratch of at least loza_ssa_decode_workspace_bytes(...) bytes, 16-byte
 *           aligned; contents on entry are ignored, on exit unspecified. It holds, per (b, query
 *           head, key split), the unnormalised fp32 partial output and four floats of softmax
 *           state. Two calls that overlap in time need two workspaces.
 * Supported (d_qk, d_v) and scale: as loza_ssa_prefill. Cache rows at or beyond seqlens[b] are
 * never read. The split count depends on the sizes only (and on LOZA_DECODE_SPLITS, see above), and
 * the merge adds the splits in a fixed order: the result is deterministic.
 * Numerics: as loza_ssa_prefill with one-term weights, except that a query with fewer than 128
 * live keys, and a query whose merged result reaches magnitude 1.97 in some column, is computed
 * from the cache rows directly in fp32 (weights not rounded at all; a rare, slower path: one
 * workgroup walks all live keys of that query).
 */
int loza_ssa_decode(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                    void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                    int d_qk, int d_v, int64_t n_sink, int64_t window, float scale,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * loza_ssa_decode for callers that cannot allocate device memory or carry a workspace around (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels,
 * the same result bits, with the partial results of the key splits in a buffer that is part of the
 * library image (LOZA_DECODE_STATIC_BYTES of device memory on every GPU the library is used on, held
 * until the process ends). No hipMalloc / hipFree, here or in anything it calls.
 *   - sizes whose workspace (loza_ssa_decode_workspace_bytes) exceeds LOZA_DECODE_STATIC_BYTES are
 *     rejected with LOZA_ERR_WORKSPACE before anything is launched; LOZA_DECODE_STATIC_BYTES covers
 *     B * Hq * splits <= 20,321 at d_v = 512 (B = 64 sequences of 64 heads in 4 splits use 16,384).
 *   - every call on a GPU uses that GPU's one buffer: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it and must be serialised by the caller. Nothing in it has to
 *     survive or be cleared between calls.
 * All other arguments, errors and numerics: as loza_ssa_decode.
 */
#define LOZA_DECODE_STATIC_BYTES (40u << 20)
int loza_ssa_decode_static(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                           void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                           int d_qk, int d_v, int64_t n_sink, int64_t window, float scale, void *stream);

/* Host-only (ours). Bytes of workspace loza_ssa_decode needs for these sizes (0 on invalid sizes). */
size_t loza_ssa_decode_workspace_bytes(int B, int Hq, int Hkv, int64_t S_max, int d_v,
                                       int64_t n_sink, int64_t window);

/* Host-only (ours). Number of key splits loza_ssa_decode uses for these sizes (0 on invalid sizes). */
int loza_ssa_decode_num_splits(int B, int Hq, int Hkv, int64_t S_max, int64_t n_sink, int64_t window);

/*
 * Host-only, no GPU involved: the live set of query i as at most two half-open key ranges,
 * [0, *sink_end) and [*win_begin, *win_end), disjoint and in order (sink_end <= win_begin).
 * This is the arithmetic the kernels enumerate tiles with (Eq. 4's pattern, "single uniform
 * schedule" of the Desiderata section: no per-head metadata).
 */
int loza_ssa_live_ranges(int64_t i, int64_t n_sink, int64_t window,
                         int64_t *sink_end, int64_t *win_begin, int64_t *win_end);

/* Host-only (ours). Live (query, key) pairs of a causal length-S prefill: the sum over i of |live(i)|
 * for the live sets of Eq. 4 as defined at the top of this file. This is the pair count the
 * benchmark's FLOP figure is built on ("compute per query stays constant": Architecture section). */
int64_t loza_ssa_live_pairs(int64_t S, int64_t n_sink, int64_t window);

/*
 * The same operation under the block-granular pattern the paper parametrises SSA with
 * (Architecture section, after Eq. 4: number of sink blocks s, number of local blocks l, block
 * size b; Training section: b = 128, s = 1, l = 7, at most 1,024 live tokens). Keys and queries
 * are cut into blocks of `block` tokens; the query at position i, in block qb = i / block, sees
 *     live(i) = { j : j <= i  and ( j / block < sink_blocks  or  qb - j / block < local_blocks ) }
 * i.e. the whole sink blocks and the local_blocks most recent blocks, its own block counted as one
 * of them and cut at the query. |live(i)| runs through (s + l - 1) b + 1 ... (s + l) b within each
 * block once i >= (s + l) b. With block == 1 this is the token-granular pattern with
 * n_sink = sink_blocks and window = local_blocks.
 * sink_blocks >= 0, local_blocks >= 1, block >= 1 (else LOZA_ERR_SHAPE); everything else
 * (layouts, supported shapes, numerics, error behaviour) as for the token-granular twin.
 * loza_ssa_decode_blocks takes a workspace of
 *     loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, sink_blocks * block, local_blocks * block)
 * bytes (products saturating at INT64_MAX) and uses the split count of the same sizes.
 */
int loza_ssa_prefill_blocks(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                            int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

int loza_ssa_prefill_blocks_f32(const float *q, const float *k, const float *v, float *out, float *lse,
                                int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

int loza_ssa_decode_blocks(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                           void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                           int d_qk, int d_v, int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * SSA "extend": q_len new query tokens per sequence against that sequence's KV cache, which already
 * holds their keys and values (chunked prefill, verification of speculated tokens: the engine side of
 * the paper's Efficiency section). Query r of sequence b sits at position seqlens[b] - q_len + r and
 * sees the live set of that position; q_len == 1 is what loza_ssa_decode computes.
 *   q       [B, q_len, Hq, d_qk] bf16
 *   kcache  [B, S_max, Hkv, d_qk] bf16     vcache [B, S_max, Hkv, d_v] bf16 (or vcache == kcache)
 *   seqlens [B] int32 (device): valid cache rows, the q_len new tokens included; a value above
 *           S_max is cut to it. Queries whose position would be negative (seqlens[b] < q_len)
 *           give out = 0, lse = -inf.
 *   out     [B, q_len, Hq, d_v] bf16       lse [B, Hq, q_len] fp32
 * 1 <= q_len <= S_max (else LOZA_ERR_SHAPE). No workspace: the prefill kernel runs over the q_len
 * positions (no split over keys), so it suits q_len * Hq / Hkv of a few hundred rows and more.
 * Supported shapes, numerics, errors: as loza_ssa_prefill / loza_ssa_prefill_blocks.
 */
int loza_ssa_extend(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens, void *out, float *lse,
                    int B, int Hq, int Hkv, int64_t S_max, int q_len, int d_qk, int d_v,
                    int64_t n_sink, int64_t window, float scale, void *stream);

int loza_ssa_extend_blocks(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens, void *out,
                           float *lse, int B, int Hq, int Hkv, int64_t S_max, int q_len, int d_qk, int d_v,
                           int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

/*
 * loza_ssa_extend / loza_ssa_extend_blocks against a paged cache: k_pages, v_pages, block_table,
 * num_pages, page_size, max_pages_per_seq as for loza_ssa_decode_paged below (same conditions on
 * page_size and on the table entries), q, seqlens, out, lse as for loza_ssa_extend, with
 * max_pages_per_seq * page_size in the place of S_max.
 */
int loza_ssa_extend_paged(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                          const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                          int64_t num_pages, int page_size, int max_pages_per_seq, int q_len, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale, void *stream);

int loza_ssa_extend_paged_blocks(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                                 const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                                 int64_t num_pages, int page_size, int max_pages_per_seq, int q_len, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

/*
 * SSA decode against a PAGED KV cache (the cache layout of a serving engine; the paper's
 * Efficiency section measures its decode kernel inside one). The rows of sequence b live in pages
 * of `page_size` rows: logical row j is row j % page_size of physical page
 * block_table[b * max_pages_per_seq + j / page_size].
 *   k_pages [num_pages, page_size, Hkv, d_qk] bf16   v_pages [num_pages, page_size, Hkv, d_v] bf16
 *           (or v_pages == k_pages: values are the first d_v elements of the key rows)
 *   block_table [B, max_pages_per_seq] int32 (device). Only the entries of pages that hold a live
 *           key are read (sink pages and the pages of the window); they must lie in [0, num_pages).
 *           An entry outside that range is cut to it: no fault, but the wrong rows.
 *   seqlens [B] int32 (device), 0 <= seqlens[b] <= max_pages_per_seq * page_size.
 *   page_size: a power of two >= 32 (else LOZA_ERR_SHAPE).
 *   workspace: loza_ssa_decode_workspace_bytes(B, Hq, Hkv, max_pages_per_seq * page_size, d_v, n_sink, window)
 *           bytes (for the _blocks form with sink_blocks * block and local_blocks * block).
 * Everything else as loza_ssa_decode / loza_ssa_decode_blocks; the result is the same bits as for
 * the same rows in a contiguous cache.
 */
int loza_ssa_decode_paged(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                          const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                          int64_t num_pages, int page_size, int max_pages_per_seq, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale,
                          void *workspace, size_t workspace_bytes, void *stream);

int loza_ssa_decode_paged_blocks(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                                 const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                                 int64_t num_pages, int page_size, int max_pages_per_seq, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Calibration forward (paper: Architecture section, Eq. 3): the layer output with the learnable
 * mixing factor alpha in [0, 1] between full attention O and streaming sparse attention O',
 *     out = alpha * O + (1 - alpha) * O'
 * for the block-granular pattern (block == 1: token-granular with n_sink = sink_blocks and
 * window = local_blocks). Two prefill passes (all causal keys; the sparse pattern) leave their
 * unrounded fp32 outputs in the workspace; a third kernel mixes them and rounds once to bf16.
 *   out        [B, S, Hq, d_v] bf16  the blend
 *   out_full   NULL or [B, S, Hq, d_v] bf16: O itself      out_sparse  NULL or the same for O'
 *              (alpha's gradient is the inner product of the incoming gradient with O - O')
 *   lse_full, lse_sparse [B, Hq, S] fp32: the log-sum-exp of either pass
 *   workspace  loza_ssa_calibration_workspace_bytes(B, Hq, S, d_v) bytes, 16-byte aligned
 * alpha outside [0, 1] or NaN: LOZA_ERR_SHAPE. Everything else as loza_ssa_prefill_blocks.
 */
int loza_ssa_prefill_calibration_blocks(const void *q, const void *k, const void *v,
                                        void *out, void *out_full, void *out_sparse, float *lse_full, float *lse_sparse,
                                        int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                        int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                        float alpha, float scale, void *workspace, size_t workspace_bytes, void *stream);

/* Host-only (ours). Workspace bytes of loza_ssa_prefill_calibration_blocks (0 on invalid sizes). */
size_t loza_ssa_calibration_workspace_bytes(int B, int Hq, int64_t S, int d_v);

/*
 * Gradient of the calibration blend with respect to alpha (Architecture section, Eq. 3): the blend is
 * alpha O + (1 - alpha) O', so d(alpha) = sum over every element of dout * (O - O').
 *   dout, out_full, out_sparse: n bf16 elements each (device, 16-byte aligned): the gradient arriving
 *       at the blend and the two outputs loza_ssa_prefill_calibration_blocks wrote; n >= 8, a multiple of 8
 *   dalpha: one float on the device (overwritten)
 *   workspace: loza_ssa_calibration_alpha_grad_workspace_bytes(n) bytes of device memory (host-only
 *       helper, ours; 0 for an n the call rejects), 16-byte aligned, contents ignored
 * Products and sums in fp64 in a fixed order (deterministic), one rounding to fp32 at the end.
 */
int loza_ssa_calibration_alpha_grad(const void *dout, const void *out_full, const void *out_sparse, float *dalpha, int64_t n,
                                    void *workspace, size_t workspace_bytes, void *stream);
size_t loza_ssa_calibration_alpha_grad_workspace_bytes(int64_t n);

/*
 * SSA backward: the gradients of loza_ssa_prefill's output with respect to q, k and v, over live
 * (query, key) pairs only. This is what training a sparsified model differentiates (paper:
 * Architecture section, Eq. 4 and its Training paragraph; the paper states no formulas, they are the
 * chain rule of a softmax):
 *     p_ij = exp(scale q_i.k_j - lse_i) for live j,  D_i = dout_i . out_i,
 *     dv_j = sum_i p_ij dout_i,  ds_ij = p_ij (dout_i . v_j - D_i),
 *     dq_i = scale sum_j ds_ij k_j,  dk_j = scale sum_i ds_ij q_i,
 * the sums over i taking every query head of the key's group.
 *   q, k, v     as loza_ssa_prefill (bf16; v == k allowed)
 *   out  [B, S, Hq, d_v] bf16 and lse [B, Hq, S] fp32: what loza_ssa_prefill returned for q, k, v
 *   dout [B, S, Hq, d_v] bf16: gradient arriving at out
 *   dq   [B, S, Hq, d_qk] bf16      dk [B, S, Hkv, d_qk] bf16      dv [B, S, Hkv, d_v] bf16
 *        When v == k, the one tensor serves as keys and (its first d_v columns) as values; dk then
 *        receives the gradient with respect to that tensor (dk with dv added to its first d_v
 *        columns) and dv is ignored (may be NULL).
 *   workspace: loza_ssa_backward_workspace_bytes(...) bytes of device memory, 16-byte aligned;
 *        contents on entry are ignored. Two calls that overlap in time need two workspaces.
 * Supported: the (d_qk, d_v) pairs of loza_ssa_prefill, scale > 0, and Hq / Hkv a power of two up to
 * 32 or a multiple of 32 (else LOZA_ERR_UNSUPPORTED). Arithmetic: bf16 matrix-core operands (q, k,
 * v, dout, and p and ds rounded to bf16), fp32 accumulation, one rounding of each result to bf16.
 * Sums run in a fixed order: the result is deterministic. No output aliases an input.
 */
int loza_ssa_backward(const void *q, const void *k, const void *v, const void *out, const float *lse,
                      const void *dout, void *dq, void *dk, void *dv,
                      int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                      int64_t n_sink, int64_t window, float scale,
                      void *workspace, size_t workspace_bytes, void *stream);

/* The same under the block-granular pattern of loza_ssa_prefill_blocks. */
int loza_ssa_backward_blocks(const void *q, const void *k, const void *v, const void *out, const float *lse,
                             const void *dout, void *dq, void *dk, void *dv,
                             int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                             int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * fp32 twins of loza_ssa_decode and loza_ssa_decode_blocks (same definition: the query of sequence b
 * sits at position seqlens[b] - 1 of its cache; Architecture section, Eq. 2 / Eq. 4): fp32 in, fp32
 * arithmetic, fp32 out, the layouts of the bf16 calls with float elements. Any d_qk, d_v in [1, 256];
 * vcache may alias kcache with d_v <= d_qk; a length beyond S_max is cut to it; an empty cache gives
 * out = 0 and lse = -inf. No workspace (one wavefront per query walks all of its live keys).
 */
int loza_ssa_decode_f32(const float *q, const float *kcache, const float *vcache, const int32_t *seqlens, float *out, float *lse,
                        int B, int Hq, int Hkv, int64_t S_max, int d_qk, int d_v,
                        int64_t n_sink, int64_t window, float scale, void *stream);
int loza_ssa_decode_blocks_f32(const float *q, const float *kcache, const float *vcache, const int32_t *seqlens, float *out,
                               float *lse, int B, int Hq, int Hkv, int64_t S_max, int d_qk, int d_v,
                               int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

/*
 * fp32 twins of loza_ssa_backward and loza_ssa_backward_blocks (the gradient of the paper's Eq. 4, as
 * above): fp32 in, fp32 arithmetic, fp32 out, the layouts of the bf16 calls with float elements; out
 * and lse are what loza_ssa_prefill_f32 returned. Any d_qk, d_v in [1, 256], any Hq / Hkv; v may alias
 * k with d_v <= d_qk (dk then receives the whole gradient of the shared tensor and dv is ignored);
 * scale finite, any sign. No workspace; deterministic (every sum runs in a fixed order). Plain vector
 * arithmetic (no matrix cores): the small-shape check of the method, not a fast path.
 */
int loza_ssa_backward_f32(const float *q, const float *k, const float *v, const float *out, const float *lse,
                          const float *dout, float *dq, float *dk, float *dv,
                          int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale, void *stream);
int loza_ssa_backward_blocks_f32(const float *q, const float *k, const float *v, const float *out, const float *lse,
                                 const float *dout, float *dq, float *dk, float *dv,
                                 int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream);

/* Host-only (ours). Workspace bytes of loza_ssa_backward / loza_ssa_backward_blocks for these sizes
 * (v_aliases_k: nonzero when v == k will be passed); 0 on sizes the call would reject. */
size_t loza_ssa_backward_workspace_bytes(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                         int64_t n_sink, int64_t window, int v_aliases_k);
size_t loza_ssa_backward_workspace_bytes_blocks(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                                int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                                int v_aliases_k);

/* Host-only twins (ours) of loza_ssa_live_ranges / loza_ssa_live_pairs for the block-granular pattern
 * (Architecture section after Eq. 4: sink blocks, local blocks, block size). */
int loza_ssa_live_ranges_blocks(int64_t i, int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                int64_t *sink_end, int64_t *win_begin, int64_t *win_end);
int64_t loza_ssa_live_pairs_blocks(int64_t S, int64_t sink_blocks, int64_t local_blocks, int64_t block);

/* Host-only (ours). Static string naming a status code. */
const char *loza_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* LOZA_SSA_H */
