// C ABI of the SSA library: argument validation, host-side schedule arithmetic, dispatch.
// Every check runs before the first HIP call, so a rejected call launches nothing.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include <mutex>

#include "../../include/loza_ssa.h"
#include "ssa_kernels.h"

// Scratch memory of loza_ssa_decode_static: the split kernel's partial results, in the place of a
// caller's workspace. One copy per GPU, at an address of its own on each; the name below is only a
// host-side handle for hipGetSymbolAddress and is never passed to a kernel.
static __device__ __align__(256) unsigned char scratch[LOZA_DECODE_STATIC_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];      // device address of `scratch` on device d (nullptr: not asked yet)

// Device address of the scratch array on the current device (asked once per device, then kept).
int scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LOZA_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void *a = nullptr;
        if (hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)) != hipSuccess || a == nullptr) return LOZA_ERR_HIP;
        scratch_ptr[dev] = a;
    }
    *ptr = scratch_ptr[dev];
    return LOZA_OK;
}

constexpr int kComputeUnits = 256;              // MI355X
constexpr int64_t kMaxSeq = 2147483647LL - 128;  // positions are 32-bit inside the kernels
constexpr int kMaxSplits = 64;                   // key splits of a decode query, at most

inline bool aligned16(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0; }

// window / n_sink cut to what can matter for sequences of at most S keys
inline int clamp_to(int64_t x, int64_t S) { return (int)(x < S ? x : S); }

int check_common(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v, int64_t n_sink, int64_t window, float scale)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || S < 1 || d_qk < 1 || d_v < 1) return LOZA_ERR_SHAPE;
    if (Hq % Hkv != 0) return LOZA_ERR_SHAPE;
    if (S > kMaxSeq) return LOZA_ERR_SHAPE;
    if (n_sink < 0 || window < 1) return LOZA_ERR_SHAPE;
    if (!(scale == scale) || isinf(scale)) return LOZA_ERR_SHAPE;
    return LOZA_OK;
}

int decode_splits(int B, int Hq, int Hkv, int64_t S_max, int64_t n_sink, int64_t window)
{
    const int G = Hq / Hkv;
    const int rows = loza::decode_rows_per_tile();
    const int64_t base = (int64_t)B * Hkv * ((G + rows - 1) / rows);
    // both terms are cut to S_max before they are added: either may be INT64_MAX
    int64_t live = (n_sink < S_max ? n_sink : S_max) + (window < S_max ? window : S_max);
    if (live > S_max) live = S_max;
    const int64_t tiles = (live + 63) / 64 + 2;
    int64_t n = (kComputeUnits + base - 1) / base;  // one workgroup per compute unit at least
    // LOZA_DECODE_SPLITS (documented in the header): another split count, for tests and experiments
    if (const char *env = getenv("LOZA_DECODE_SPLITS")) {
        const long v = strtol(env, nullptr, 10);
        if (v >= 1 && v <= kMaxSplits) n = v;
    }
    if (n > tiles) n = tiles;
    if (n > kMaxSplits) n = kMaxSplits;
    if (n < 1) n = 1;
    return (int)n;
}

// The pattern as the kernels take it: sink in tokens, window in blocks of `block` tokens, both cut
// to what can matter for S keys. The token-granular entry points use block = 1.
struct Pattern {
    int n_sink, window, block;
};

inline int64_t sat_mul(int64_t a, int64_t b) { return (a != 0 && b > INT64_MAX / a) ? INT64_MAX : a * b; }

Pattern token_pattern(int64_t n_sink, int64_t window, int64_t S)
{
    return Pattern{clamp_to(n_sink, S), clamp_to(window, S), 1};
}

// block-granular: sink_blocks >= 0, local_blocks >= 1, block >= 1 (checked by the caller)
Pattern block_pattern(int64_t sink_blocks, int64_t local_blocks, int64_t block, int64_t S)
{
    const int64_t b = block < S ? block : S;  // one block already covers everything
    if (block >= S) return Pattern{sink_blocks > 0 ? (int)S : 0, 1, (int)b};
    return Pattern{clamp_to(sat_mul(sink_blocks, block), S), clamp_to(local_blocks, S / block + 1), (int)b};
}

int check_blocks(int64_t sink_blocks, int64_t local_blocks, int64_t block)
{
    return (sink_blocks < 0 || local_blocks < 1 || block < 1) ? LOZA_ERR_SHAPE : LOZA_OK;
}

// The reference maximum of the online softmax is the exact running maximum over the first 8 key
// tiles of a row tile and afterwards moves only when exceeded by more than 2^8 (fp32 has the headroom).
void set_rescale_policy(loza::FwdParams &p)
{
    p.exact_tiles = 8;
    p.lazy_log2 = 8.0f;
}

}  // namespace

extern "C" {

const char *loza_status_str(int status)
{
    switch (status) {
    case LOZA_OK: return "LOZA_OK";
    case LOZA_ERR_NULL: return "LOZA_ERR_NULL: a required pointer is NULL";
    case LOZA_ERR_SHAPE: return "LOZA_ERR_SHAPE: sizes out of range or inconsistent";
    case LOZA_ERR_UNSUPPORTED: return "LOZA_ERR_UNSUPPORTED: no kernel for this (dtype, d_qk, d_v)";
    case LOZA_ERR_WORKSPACE: return "LOZA_ERR_WORKSPACE: workspace missing or too small";
    case LOZA_ERR_HIP: return "LOZA_ERR_HIP: a HIP call failed";
    case LOZA_ERR_ALIGN: return "LOZA_ERR_ALIGN: a base pointer is not 16-byte aligned";
    default: return "unknown loza status";
    }
}

int loza_ssa_live_ranges(int64_t i, int64_t n_sink, int64_t window,
                         int64_t *sink_end, int64_t *win_begin, int64_t *win_end)
{
    if (!sink_end || !win_begin || !win_end) return LOZA_ERR_NULL;
    if (i < 0 || i == INT64_MAX || n_sink < 0 || window < 1) return LOZA_ERR_SHAPE;  // i + 1 is returned
    const int64_t se = n_sink < i + 1 ? n_sink : i + 1;
    int64_t wb = window > i ? 0 : i - window + 1;
    if (wb < se) wb = se;  // a key in both sets is used once
    *sink_end = se;
    *win_begin = wb;
    *win_end = i + 1;
    return LOZA_OK;
}

int loza_ssa_live_ranges_blocks(int64_t i, int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                int64_t *sink_end, int64_t *win_begin, int64_t *win_end)
{
    if (!sink_end || !win_begin || !win_end) return LOZA_ERR_NULL;
    if (i < 0 || i == INT64_MAX || check_blocks(sink_blocks, local_blocks, block) != LOZA_OK) return LOZA_ERR_SHAPE;
    const int64_t sink_tokens = sat_mul(sink_blocks, block);
    const int64_t se = sink_tokens < i + 1 ? sink_tokens : i + 1;
    const int64_t qb = i / block;
    int64_t wb = local_blocks > qb ? 0 : (qb - local_blocks + 1) * block;
    if (wb < se) wb = se;
    *sink_end = se;
    *win_begin = wb;
    *win_end = i + 1;
    return LOZA_OK;
}

int64_t loza_ssa_live_pairs_blocks(int64_t S, int64_t sink_blocks, int64_t local_blocks, int64_t block)
{
    if (S < 1 || S > kMaxSeq || check_blocks(sink_blocks, local_blocks, block) != LOZA_OK) return -1;
    // query block by query block: inside one block the window start is fixed and |live(i)| grows by one
    const int64_t sink_tokens = sat_mul(sink_blocks, block);
    if (block > S) block = S;  // one block already holds every position (and i0 + block cannot overflow)
    int64_t pairs = 0;
    for (int64_t i0 = 0; i0 < S; i0 += block) {
        const int64_t i1 = (i0 + block < S ? i0 + block : S) - 1;  // last query of the block
        const int64_t qb = i0 / block;
        const int64_t wb = local_blocks > qb ? 0 : (qb - local_blocks + 1) * block;
        const int64_t n = i1 - i0 + 1;
        if (wb <= sink_tokens) {
            pairs += n * (i0 + 1) + n * (n - 1) / 2;                       // everything up to the query
        } else {
            pairs += n * (sink_tokens + i0 + 1 - wb) + n * (n - 1) / 2;    // sink + [wb, i]
        }
    }
    return pairs;
}

int64_t loza_ssa_live_pairs(int64_t S, int64_t n_sink, int64_t window)
{
    if (S < 1 || S > kMaxSeq || n_sink < 0 || window < 1) return -1;
    // |live(i)| = min(i + 1, T), T = n_sink + window (saturating)
    const int64_t T = (window >= S || n_sink >= S || n_sink + window >= S) ? S : n_sink + window;
    return T * (T + 1) / 2 + (S - T) * T;
}

// Paged cache description (block_table == nullptr: contiguous cache of S_max rows per sequence).
struct Paging {
    const int32_t *block_table;
    int64_t num_pages;
    int page_size, max_pages;
};

// Checks a paging description and gives log2(page_size) and the capacity per sequence in rows.
static int check_paging(const Paging &pg, int *page_shift, int64_t *capacity)
{
    if (!pg.block_table) return LOZA_ERR_NULL;
    // pages hold a power-of-two number of rows that key tiles (32 rows) divide
    if (pg.page_size < 32 || (pg.page_size & (pg.page_size - 1)) != 0) return LOZA_ERR_SHAPE;
    if (pg.num_pages < 1 || pg.num_pages > 2147483647LL || pg.max_pages < 1) return LOZA_ERR_SHAPE;
    if ((int64_t)pg.max_pages * pg.page_size > kMaxSeq) return LOZA_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(pg.block_table) & 3u) return LOZA_ERR_ALIGN;
    int s = 0;
    while ((1 << s) < pg.page_size) ++s;
    *page_shift = s;
    *capacity = (int64_t)pg.max_pages * pg.page_size;
    return LOZA_OK;
}

static int prefill_bf16(const void *q, const void *k, const void *v, void *out, float *lse,
                        int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                        int64_t sink, int64_t local, int64_t block, bool blocks, float scale, void *stream,
                        float *out_f32 = nullptr, bool validate_only = false,
                        const int32_t *seqlens = nullptr, int64_t q_len = 0, const Paging *paging = nullptr)
{
    // seqlens != nullptr: "extend" form, q_len queries per sequence against a cache of S rows
    // (with a paging description: of max_pages * page_size rows behind a block table)
    const bool extend = seqlens != nullptr;
    if (!q || !k || !v || (!out && !out_f32) || !lse) return LOZA_ERR_NULL;
    int page_shift = 0;
    if (paging) {
        if (!extend) return LOZA_ERR_SHAPE;
        if (int rc = check_paging(*paging, &page_shift, &S)) return rc;
    }
    if (extend && (q_len < 1 || q_len > S || (reinterpret_cast<uintptr_t>(seqlens) & 3u))) return q_len < 1 || q_len > S ? LOZA_ERR_SHAPE : LOZA_ERR_ALIGN;
    if (int rc = check_common(B, Hq, Hkv, S, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    if (!(scale > 0.f)) return LOZA_ERR_SHAPE;  // the row maximum is taken before the scaling
    const bool alias = (v == k);
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (!loza::bf16_shape_supported(d_qk, d_v, alias)) return LOZA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse)) return LOZA_ERR_ALIGN;
    const int G = Hq / Hkv;
    const int rows = loza::prefill_rows_per_tile();
    const int64_t row_tiles = ((extend ? q_len : S) * G + rows - 1) / rows;
    if (row_tiles * Hkv * B > 2147483647LL) return LOZA_ERR_SHAPE;
    if (validate_only) return LOZA_OK;

    loza::FwdParams p{};
    p.q = (const uint16_t *)q; p.k = (const uint16_t *)k; p.v = (const uint16_t *)v;
    p.out = (uint16_t *)out; p.out_f32 = out_f32; p.lse = lse;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.S = S;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S) : token_pattern(sink, local, S);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale_log2 = scale * 1.44269504088896340736f;
    p.row_tiles = (int)row_tiles; p.n_splits = 1;
    set_rescale_policy(p);
    if (extend) {
        p.seqlens = seqlens; p.q_len = (int)q_len;
        if (paging) {
            p.block_table = paging->block_table;
            p.page_shift = page_shift; p.max_pages = paging->max_pages; p.num_pages = (int)paging->num_pages;
        }
        return loza::launch_extend_bf16(p, d_qk, d_v, alias, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
    }
    return loza::launch_prefill_bf16(p, d_qk, d_v, alias, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_extend(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens, void *out, float *lse,
                    int B, int Hq, int Hkv, int64_t S_max, int q_len, int d_qk, int d_v,
                    int64_t n_sink, int64_t window, float scale, void *stream)
{
    if (!seqlens) return LOZA_ERR_NULL;
    return prefill_bf16(q, kcache, vcache, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, 1, false, scale, stream,
                        nullptr, false, seqlens, q_len);
}

int loza_ssa_extend_paged(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                          const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                          int64_t num_pages, int page_size, int max_pages_per_seq, int q_len, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale, void *stream)
{
    if (!seqlens) return LOZA_ERR_NULL;
    const Paging pg{block_table, num_pages, page_size, max_pages_per_seq};
    return prefill_bf16(q, k_pages, v_pages, out, lse, B, Hq, Hkv, 1, d_qk, d_v, n_sink, window, 1, false, scale, stream,
                        nullptr, false, seqlens, q_len, &pg);
}

int loza_ssa_extend_paged_blocks(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                                 const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                                 int64_t num_pages, int page_size, int max_pages_per_seq, int q_len, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    if (!seqlens) return LOZA_ERR_NULL;
    const Paging pg{block_table, num_pages, page_size, max_pages_per_seq};
    return prefill_bf16(q, k_pages, v_pages, out, lse, B, Hq, Hkv, 1, d_qk, d_v, sink_blocks, local_blocks, block, true,
                        scale, stream, nullptr, false, seqlens, q_len, &pg);
}

int loza_ssa_extend_blocks(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens, void *out,
                           float *lse, int B, int Hq, int Hkv, int64_t S_max, int q_len, int d_qk, int d_v,
                           int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    if (!seqlens) return LOZA_ERR_NULL;
    return prefill_bf16(q, kcache, vcache, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, sink_blocks, local_blocks, block, true,
                        scale, stream, nullptr, false, seqlens, q_len);
}

int loza_ssa_prefill(const void *q, const void *k, const void *v, void *out, float *lse,
                     int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                     int64_t n_sink, int64_t window, float scale, void *stream)
{
    return prefill_bf16(q, k, v, out, lse, B, Hq, Hkv, S, d_qk, d_v, n_sink, window, 1, false, scale, stream);
}

int loza_ssa_prefill_blocks(const void *q, const void *k, const void *v, void *out, float *lse,
                            int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                            int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    return prefill_bf16(q, k, v, out, lse, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true, scale, stream);
}

static int prefill_f32(const float *q, const float *k, const float *v, float *out, float *lse,
                       int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                       int64_t sink, int64_t local, int64_t block, bool blocks, float scale, void *stream)
{
    if (!q || !k || !v || !out || !lse) return LOZA_ERR_NULL;
    if (int rc = check_common(B, Hq, Hkv, S, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    const bool alias = (v == k);
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (d_qk > 256 || d_v > 256) return LOZA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse)) return LOZA_ERR_ALIGN;
    if (((int64_t)B * S * Hq + 3) / 4 > 2147483647LL) return LOZA_ERR_SHAPE;

    loza::F32Params p{};
    p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.S = S; p.d_qk = d_qk; p.d_v = d_v;
    p.k_row = d_qk; p.v_row = alias ? d_qk : d_v;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S) : token_pattern(sink, local, S);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale = scale;
    return loza::launch_prefill_f32(p, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

static int decode_f32(const float *q, const float *kcache, const float *vcache, const int32_t *seqlens, float *out, float *lse,
                      int B, int Hq, int Hkv, int64_t S_max, int d_qk, int d_v,
                      int64_t sink, int64_t local, int64_t block, bool blocks, float scale, void *stream)
{
    if (!q || !kcache || !vcache || !seqlens || !out || !lse) return LOZA_ERR_NULL;
    if (int rc = check_common(B, Hq, Hkv, S_max, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    const bool alias = (vcache == kcache);
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (d_qk > 256 || d_v > 256) return LOZA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(kcache) || !aligned16(vcache) || !aligned16(out) ||
        (reinterpret_cast<uintptr_t>(seqlens) & 3u) || (reinterpret_cast<uintptr_t>(lse) & 3u))
        return LOZA_ERR_ALIGN;
    if (((int64_t)B * Hq + 3) / 4 > 2147483647LL) return LOZA_ERR_SHAPE;

    loza::F32Params p{};
    p.q = q; p.k = kcache; p.v = vcache; p.out = out; p.lse = lse; p.seqlens = seqlens;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.S = S_max; p.d_qk = d_qk; p.d_v = d_v;
    p.k_row = d_qk; p.v_row = alias ? d_qk : d_v;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S_max) : token_pattern(sink, local, S_max);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale = scale;
    return loza::launch_prefill_f32(p, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_decode_f32(const float *q, const float *kcache, const float *vcache, const int32_t *seqlens, float *out, float *lse,
                        int B, int Hq, int Hkv, int64_t S_max, int d_qk, int d_v,
                        int64_t n_sink, int64_t window, float scale, void *stream)
{
    return decode_f32(q, kcache, vcache, seqlens, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, 1, false, scale, stream);
}

int loza_ssa_decode_blocks_f32(const float *q, const float *kcache, const float *vcache, const int32_t *seqlens, float *out,
                               float *lse, int B, int Hq, int Hkv, int64_t S_max, int d_qk, int d_v,
                               int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    return decode_f32(q, kcache, vcache, seqlens, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, sink_blocks, local_blocks, block, true,
                      scale, stream);
}

size_t loza_ssa_calibration_workspace_bytes(int B, int Hq, int64_t S, int d_v)
{
    if (B < 1 || Hq < 1 || S < 1 || d_v < 1 || S > kMaxSeq) return 0;
    return (size_t)2 * B * S * Hq * d_v * sizeof(float);
}

int loza_ssa_prefill_calibration_blocks(const void *q, const void *k, const void *v,
                                        void *out, void *out_full, void *out_sparse, float *lse_full, float *lse_sparse,
                                        int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                        int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                        float alpha, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out || !lse_full || !lse_sparse) return LOZA_ERR_NULL;
    if (!(alpha >= 0.f && alpha <= 1.f)) return LOZA_ERR_SHAPE;
    const size_t need = loza_ssa_calibration_workspace_bytes(B, Hq, S, d_v);
    if (need == 0) return LOZA_ERR_SHAPE;
    if (!workspace || workspace_bytes < need) return LOZA_ERR_WORKSPACE;
    if (!aligned16(out) || !aligned16(workspace) || (out_full && !aligned16(out_full)) || (out_sparse && !aligned16(out_sparse)))
        return LOZA_ERR_ALIGN;
    float *o_full = (float *)workspace, *o_sparse = o_full + need / (2 * sizeof(float));
    // every argument of both passes is checked before the first launch
    if (int rc = prefill_bf16(q, k, v, nullptr, lse_full, B, Hq, Hkv, S, d_qk, d_v, 0, 1, INT64_MAX, true, scale, stream, o_full, true))
        return rc;
    if (int rc = prefill_bf16(q, k, v, nullptr, lse_sparse, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true,
                              scale, stream, o_sparse, true))
        return rc;
    // O: every causal key (one block that holds everything); O': the sparse pattern
    if (int rc = prefill_bf16(q, k, v, nullptr, lse_full, B, Hq, Hkv, S, d_qk, d_v, 0, 1, INT64_MAX, true, scale, stream, o_full))
        return rc;
    if (int rc = prefill_bf16(q, k, v, nullptr, lse_sparse, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true,
                              scale, stream, o_sparse))
        return rc;
    const int64_t n = (int64_t)B * S * Hq * d_v;  // a multiple of 8: d_v is
    return loza::launch_blend_bf16(o_full, o_sparse, alpha, (uint16_t *)out, (uint16_t *)out_full, (uint16_t *)out_sparse, n,
                                   (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

size_t loza_ssa_calibration_alpha_grad_workspace_bytes(int64_t n)
{
    if (n < 8 || n % 8 != 0) return 0;
    return (size_t)loza::alpha_grad_blocks(n) * sizeof(double);
}

int loza_ssa_calibration_alpha_grad(const void *dout, const void *out_full, const void *out_sparse, float *dalpha, int64_t n,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dout || !out_full || !out_sparse || !dalpha) return LOZA_ERR_NULL;
    const size_t need = loza_ssa_calibration_alpha_grad_workspace_bytes(n);
    if (need == 0) return LOZA_ERR_SHAPE;
    if (!workspace || workspace_bytes < need) return LOZA_ERR_WORKSPACE;
    if (!aligned16(dout) || !aligned16(out_full) || !aligned16(out_sparse) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(dalpha) & 3u))
        return LOZA_ERR_ALIGN;
    return loza::launch_alpha_grad_bf16((const uint16_t *)dout, (const uint16_t *)out_full, (const uint16_t *)out_sparse, dalpha, n,
                                        (double *)workspace, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_prefill_f32(const float *q, const float *k, const float *v, float *out, float *lse,
                         int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                         int64_t n_sink, int64_t window, float scale, void *stream)
{
    return prefill_f32(q, k, v, out, lse, B, Hq, Hkv, S, d_qk, d_v, n_sink, window, 1, false, scale, stream);
}

int loza_ssa_prefill_blocks_f32(const float *q, const float *k, const float *v, float *out, float *lse,
                                int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    return prefill_f32(q, k, v, out, lse, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true, scale, stream);
}

// ---- backward ---------------------------------------------------------------------------------------

// Host-side schedule of the key-stationary backward kernel: how many key tiles hold sink keys (their
// rows run in chunks as workgroups of their own), how long a chunk is, how many the first tile has.
static void backward_plan(loza::BwdParams &p)
{
    const int64_t n_kt = (p.S + 63) / 64;
    const int64_t sink_kt = ((int64_t)p.n_sink + 63) / 64;
    p.n_sink_kt = (int)(sink_kt < n_kt ? sink_kt : n_kt);
    // a chunk is as long as the row range of a key tile without sink keys (64 keys + the window's reach)
    const int64_t reach = (int64_t)p.window * p.block + 64 + p.block;
    int64_t ct = ((reach < p.S ? reach : p.S) * p.G + 31) / 32 + 1;
    if (ct < 64) ct = 64;
    p.chunk_tiles = (int)ct;
    int lo, hi;
    loza::bwd_key_tile_rows(p, 0, lo, hi);
    p.max_chunks = p.n_sink_kt > 0 ? (int)((hi - lo + 1 + ct - 1) / ct) : 1;
}

static int backward_fill(loza::BwdParams &p, int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                         int64_t sink, int64_t local, int64_t block, bool blocks, float scale, bool alias)
{
    if (int rc = check_common(B, Hq, Hkv, S, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    if (!(scale > 0.f)) return LOZA_ERR_SHAPE;
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (!loza::bf16_shape_supported(d_qk, d_v, alias)) return LOZA_ERR_UNSUPPORTED;
    if (!loza::bwd_group_supported(Hq / Hkv)) return LOZA_ERR_UNSUPPORTED;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.S = S;
    if (S * p.G > 2147483647LL - 64) return LOZA_ERR_SHAPE;
    p.r_pad = (S * p.G + 31) / 32 * 32;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S) : token_pattern(sink, local, S);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale = scale;
    p.scale_log2 = scale * 1.44269504088896340736f;
    backward_plan(p);
    const int64_t n_kt = (S + 63) / 64;
    const int64_t items = (int64_t)p.n_sink_kt * p.max_chunks + (n_kt - p.n_sink_kt);
    if (items * Hkv * B > 2147483647LL || ((S * p.G + 63) / 64) * Hkv * B > 2147483647LL ||
        ((int64_t)B * S * Hq + 3) / 4 > 2147483647LL)
        return LOZA_ERR_SHAPE;
    return LOZA_OK;
}

static size_t backward_bytes(const loza::BwdParams &p, int d_qk, int d_v, bool alias, size_t *part_offset)
{
    size_t stat = (size_t)p.B * p.Hkv * (size_t)p.r_pad * sizeof(float2);
    stat = (stat + 255) / 256 * 256;
    if (part_offset) *part_offset = stat;
    const size_t cols = alias ? (size_t)d_qk : (size_t)d_qk + d_v;
    const size_t part = p.max_chunks > 1 ? (size_t)p.B * p.Hkv * p.n_sink_kt * p.max_chunks * 64 * cols * sizeof(float) : 0;
    return stat + part;
}

static size_t backward_workspace(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                 int64_t sink, int64_t local, int64_t block, bool blocks, int alias)
{
    loza::BwdParams p{};
    if (backward_fill(p, B, Hq, Hkv, S, d_qk, d_v, sink, local, block, blocks, 1.0f, alias != 0) != LOZA_OK) return 0;
    return backward_bytes(p, d_qk, d_v, alias != 0, nullptr);
}

static int backward_bf16(const void *q, const void *k, const void *v, const void *out, const float *lse,
                         const void *dout, void *dq, void *dk, void *dv,
                         int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                         int64_t sink, int64_t local, int64_t block, bool blocks, float scale,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk) return LOZA_ERR_NULL;
    const bool alias = (v == k);
    if (!alias && !dv) return LOZA_ERR_NULL;
    loza::BwdParams p{};
    if (int rc = backward_fill(p, B, Hq, Hkv, S, d_qk, d_v, sink, local, block, blocks, scale, alias)) return rc;
    size_t part_offset = 0;
    const size_t need = backward_bytes(p, d_qk, d_v, alias, &part_offset);
    if (!workspace || workspace_bytes < need) return LOZA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(dout) || !aligned16(dq) ||
        !aligned16(dk) || (!alias && !aligned16(dv)) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(lse) & 3u))
        return LOZA_ERR_ALIGN;
    p.q = (const uint16_t *)q; p.k = (const uint16_t *)k; p.v = (const uint16_t *)v;
    p.out = (const uint16_t *)out; p.dout = (const uint16_t *)dout; p.lse = lse;
    p.dq = (uint16_t *)dq; p.dk = (uint16_t *)dk; p.dv = alias ? nullptr : (uint16_t *)dv;
    p.rowstat = (float2 *)workspace;
    p.part = (float *)((char *)workspace + part_offset);
    return loza::launch_backward_bf16(p, d_qk, d_v, alias, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_backward(const void *q, const void *k, const void *v, const void *out, const float *lse,
                      const void *dout, void *dq, void *dk, void *dv,
                      int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                      int64_t n_sink, int64_t window, float scale,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    return backward_bf16(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, S, d_qk, d_v, n_sink, window, 1, false, scale,
                         workspace, workspace_bytes, stream);
}

int loza_ssa_backward_blocks(const void *q, const void *k, const void *v, const void *out, const float *lse,
                             const void *dout, void *dq, void *dk, void *dv,
                             int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                             int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    return backward_bf16(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block,
                         true, scale, workspace, workspace_bytes, stream);
}

static int backward_f32(const float *q, const float *k, const float *v, const float *out, const float *lse, const float *dout,
                        float *dq, float *dk, float *dv, int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                        int64_t sink, int64_t local, int64_t block, bool blocks, float scale, void *stream)
{
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk) return LOZA_ERR_NULL;
    if (int rc = check_common(B, Hq, Hkv, S, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    const bool alias = (v == k);
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (!alias && !dv) return LOZA_ERR_NULL;
    if (d_qk > 256 || d_v > 256) return LOZA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse) || !aligned16(dout) ||
        !aligned16(dq) || !aligned16(dk) || (!alias && !aligned16(dv)))
        return LOZA_ERR_ALIGN;
    if (((int64_t)B * S * Hq + 3) / 4 > 2147483647LL) return LOZA_ERR_SHAPE;

    loza::F32BwdParams p{};
    p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse; p.dout = dout;
    p.dq = dq; p.dk = dk; p.dv = alias ? nullptr : dv;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.S = S; p.d_qk = d_qk; p.d_v = d_v;
    p.k_row = d_qk; p.v_row = alias ? d_qk : d_v;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S) : token_pattern(sink, local, S);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale = scale;
    return loza::launch_backward_f32(p, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_backward_f32(const float *q, const float *k, const float *v, const float *out, const float *lse,
                          const float *dout, float *dq, float *dk, float *dv,
                          int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale, void *stream)
{
    return backward_f32(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, S, d_qk, d_v, n_sink, window, 1, false, scale, stream);
}

int loza_ssa_backward_blocks_f32(const float *q, const float *k, const float *v, const float *out, const float *lse,
                                 const float *dout, float *dq, float *dk, float *dv,
                                 int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale, void *stream)
{
    return backward_f32(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true,
                        scale, stream);
}

size_t loza_ssa_backward_workspace_bytes(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                         int64_t n_sink, int64_t window, int v_aliases_k)
{
    return backward_workspace(B, Hq, Hkv, S, d_qk, d_v, n_sink, window, 1, false, v_aliases_k);
}

size_t loza_ssa_backward_workspace_bytes_blocks(int B, int Hq, int Hkv, int64_t S, int d_qk, int d_v,
                                                int64_t sink_blocks, int64_t local_blocks, int64_t block,
                                                int v_aliases_k)
{
    if (check_blocks(sink_blocks, local_blocks, block) != LOZA_OK) return 0;
    return backward_workspace(B, Hq, Hkv, S, d_qk, d_v, sink_blocks, local_blocks, block, true, v_aliases_k);
}

int loza_ssa_decode_num_splits(int B, int Hq, int Hkv, int64_t S_max, int64_t n_sink, int64_t window)
{
    if (check_common(B, Hq, Hkv, S_max, 1, 1, n_sink, window, 1.0f) != LOZA_OK) return 0;
    return decode_splits(B, Hq, Hkv, S_max, n_sink, window);
}

size_t loza_ssa_decode_workspace_bytes(int B, int Hq, int Hkv, int64_t S_max, int d_v,
                                       int64_t n_sink, int64_t window)
{
    if (d_v < 1) return 0;
    const int n = loza_ssa_decode_num_splits(B, Hq, Hkv, S_max, n_sink, window);
    if (n == 0) return 0;
    return (size_t)B * Hq * n * ((size_t)d_v + 4) * sizeof(float);
}

static int decode_bf16(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                       void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                       int d_qk, int d_v, int64_t sink, int64_t local, int64_t block, bool blocks, float scale,
                       void *workspace, size_t workspace_bytes, void *stream, const Paging *paging = nullptr)
{
    if (!q || !kcache || !vcache || !seqlens || !out || !lse) return LOZA_ERR_NULL;
    int page_shift = 0;
    if (paging) {
        if (int rc = check_paging(*paging, &page_shift, &S_max)) return rc;
    }
    if (int rc = check_common(B, Hq, Hkv, S_max, d_qk, d_v, sink, local, scale)) return rc;
    if (blocks) { if (int rc = check_blocks(sink, local, block)) return rc; }
    if (!(scale > 0.f)) return LOZA_ERR_SHAPE;
    // the split count and the workspace are sized by the token counts the pattern can reach
    const int64_t n_sink = blocks ? sat_mul(sink, block) : sink, window = blocks ? sat_mul(local, block) : local;
    const bool alias = (vcache == kcache);
    if (alias && d_v > d_qk) return LOZA_ERR_SHAPE;
    if (!loza::bf16_shape_supported(d_qk, d_v, alias)) return LOZA_ERR_UNSUPPORTED;
    const size_t need = loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink, window);
    if (!workspace || workspace_bytes < need) return LOZA_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(kcache) || !aligned16(vcache) || !aligned16(out) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(seqlens) & 3u) || (reinterpret_cast<uintptr_t>(lse) & 3u))
        return LOZA_ERR_ALIGN;
    const int G = Hq / Hkv;
    const int rows = loza::decode_rows_per_tile();
    const int n_splits = decode_splits(B, Hq, Hkv, S_max, n_sink, window);
    const int64_t row_tiles = (G + rows - 1) / rows;
    if (row_tiles * Hkv * B * n_splits > 2147483647LL) return LOZA_ERR_SHAPE;

    loza::FwdParams p{};
    p.q = (const uint16_t *)q; p.k = (const uint16_t *)kcache; p.v = (const uint16_t *)vcache;
    p.out = (uint16_t *)out; p.lse = lse;
    p.part_o = (float *)workspace;
    p.part_ml = (float *)workspace + (size_t)B * Hq * n_splits * d_v;
    p.seqlens = seqlens;
    if (paging) {
        p.block_table = paging->block_table;
        p.page_shift = page_shift; p.max_pages = paging->max_pages; p.num_pages = (int)paging->num_pages;
    }
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.S = S_max;
    const Pattern pat = blocks ? block_pattern(sink, local, block, S_max) : token_pattern(sink, local, S_max);
    p.n_sink = pat.n_sink; p.window = pat.window; p.block = pat.block;
    p.scale_log2 = scale * 1.44269504088896340736f;
    p.row_tiles = (int)row_tiles; p.n_splits = n_splits;
    set_rescale_policy(p);
    return loza::launch_decode_bf16(p, d_qk, d_v, alias, (hipStream_t)stream) == hipSuccess ? LOZA_OK : LOZA_ERR_HIP;
}

int loza_ssa_decode(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                    void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                    int d_qk, int d_v, int64_t n_sink, int64_t window, float scale,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_bf16(q, kcache, vcache, seqlens, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, 1, false,
                       scale, workspace, workspace_bytes, stream);
}

int loza_ssa_decode_static(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                           void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                           int d_qk, int d_v, int64_t n_sink, int64_t window, float scale, void *stream)
{
    // sizes first (no HIP call on a rejected size), then the per-device address of the scratch array
    if (check_common(B, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, scale) != LOZA_OK) return LOZA_ERR_SHAPE;
    const size_t need = loza_ssa_decode_workspace_bytes(B, Hq, Hkv, S_max, d_v, n_sink, window);
    if (need == 0) return LOZA_ERR_SHAPE;
    if (need > (size_t)LOZA_DECODE_STATIC_BYTES) return LOZA_ERR_WORKSPACE;
    void *ws = nullptr;
    if (int rc = scratch_of_current_device(&ws)) return rc;
    return decode_bf16(q, kcache, vcache, seqlens, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, n_sink, window, 1, false,
                       scale, ws, (size_t)LOZA_DECODE_STATIC_BYTES, stream);
}

int loza_ssa_decode_paged(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                          const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                          int64_t num_pages, int page_size, int max_pages_per_seq, int d_qk, int d_v,
                          int64_t n_sink, int64_t window, float scale,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    const Paging pg{block_table, num_pages, page_size, max_pages_per_seq};
    return decode_bf16(q, k_pages, v_pages, seqlens, out, lse, B, Hq, Hkv, 1, d_qk, d_v, n_sink, window, 1, false,
                       scale, workspace, workspace_bytes, stream, &pg);
}

int loza_ssa_decode_paged_blocks(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                                 const int32_t *seqlens, void *out, float *lse, int B, int Hq, int Hkv,
                                 int64_t num_pages, int page_size, int max_pages_per_seq, int d_qk, int d_v,
                                 int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    const Paging pg{block_table, num_pages, page_size, max_pages_per_seq};
    return decode_bf16(q, k_pages, v_pages, seqlens, out, lse, B, Hq, Hkv, 1, d_qk, d_v, sink_blocks, local_blocks,
                       block, true, scale, workspace, workspace_bytes, stream, &pg);
}

int loza_ssa_decode_blocks(const void *q, const void *kcache, const void *vcache, const int32_t *seqlens,
                           void *out, float *lse, int B, int Hq, int Hkv, int64_t S_max,
                           int d_qk, int d_v, int64_t sink_blocks, int64_t local_blocks, int64_t block, float scale,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_bf16(q, kcache, vcache, seqlens, out, lse, B, Hq, Hkv, S_max, d_qk, d_v, sink_blocks, local_blocks,
                       block, true, scale, workspace, workspace_bytes, stream);
}

}  // extern "C"
