// Internal interface between the C-ABI translation unit and the kernel translation units.
#ifndef LOZA_SSA_KERNELS_H
#define LOZA_SSA_KERNELS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace loza {

// Arguments of the bf16 forward kernels. `S` is the sequence length of a prefill, or the row
// count (stride) of each sequence's cache in a decode. The live set of query i is
//   { j <= i : j < n_sink  or  j >= max(0, i / block - window + 1) * block },
// n_sink in tokens, window in blocks of `block` tokens (block = 1: the token-granular pattern, the
// window then counts tokens). n_sink and window are already cut by the host to what can matter
// for S keys (a window that covers S keys or more is "infinite").
struct FwdParams {
    const uint16_t *q, *k, *v;
    uint16_t *out;
    float *out_f32;  // prefill only: when set, the output goes here unrounded instead of to `out`
    float *lse;
    float *part_o;   // decode: [B, Hq, n_splits, d_v] unnormalised partial outputs
    float *part_ml;  // decode: [B, Hq, n_splits, 4]   reference max (log2 domain), sum, rounded sum, pad
    const int32_t *seqlens;
    // paged decode cache (else nullptr): logical page j >> page_shift of sequence b is physical page
    // block_table[b * max_pages + (j >> page_shift)] of k / v, which are then [num_pages, 2^page_shift, Hkv, d]
    const int32_t *block_table;
    int page_shift, max_pages, num_pages;
    int B, Hq, Hkv, G;
    int64_t S;
    int n_sink, window, block;
    float scale_log2;  // scale * log2(e)
    int row_tiles;     // workgroup tiles per (batch, kv head) in this launch
    int rt_begin;      // first of them
    int n_splits;      // decode only
    int q_len;         // extend prefill: queries per sequence (0: plain prefill); keys valid up to seqlens[b]
    int all_precise;   // prefill / extend: every tile takes the two-term pass (set by the launcher from the pattern)
    int exact_tiles;   // tiles over which the reference maximum is the exact running maximum
    float lazy_log2;   // afterwards it moves only when exceeded by this much (log2 units)
};

bool bf16_shape_supported(int d_qk, int d_v, bool alias);
int prefill_rows_per_tile();
int decode_rows_per_tile();
hipError_t launch_prefill_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream);
hipError_t launch_extend_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream);
hipError_t launch_decode_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream);
hipError_t launch_blend_bf16(const float *o_full, const float *o_sparse, float alpha, uint16_t *out,
                             uint16_t *out_full, uint16_t *out_sparse, int64_t n, hipStream_t stream);
// d(alpha) of the blend: sum of dout * (O - O') over n bf16 elements (n a multiple of 8); `partial`
// holds alpha_grad_blocks(n) doubles of scratch
int alpha_grad_blocks(int64_t n);
hipError_t launch_alpha_grad_bf16(const uint16_t *dout, const uint16_t *o_full, const uint16_t *o_sparse, float *dalpha, int64_t n,
                                  double *partial, hipStream_t stream);

// Arguments of the bf16 backward kernels. Pattern fields as in FwdParams.
struct BwdParams {
    const uint16_t *q, *k, *v, *out, *dout;
    const float *lse;
    uint16_t *dq, *dk, *dv;   // dv is unused when v aliases k (dk then holds the gradient of the shared tensor)
    float2 *rowstat;          // workspace: [B, Hkv, r_pad] (lse * log2(e), dO . O), row index i * G + head-in-group
    float *part;              // workspace: [B, Hkv, n_sink_kt, max_chunks, 64, columns] fp32 partial dK | dV
    int B, Hq, Hkv, G;
    int64_t S;
    int64_t r_pad;            // S * G rounded up to a multiple of 32
    int n_sink, window, block;
    float scale, scale_log2;
    int n_sink_kt;            // key tiles (of 64 keys) that hold at least one sink key
    int chunk_tiles;          // row tiles (of 32 rows) per chunk of such a key tile
    int max_chunks;           // chunks of the first key tile (the one with most rows)
};

// Row tiles (32 rows each, row = position * G + head-in-group) that can see a key of key tile kt
// (64 keys): from the tile's first key on (causality) to the last position whose window still holds
// the tile's last key, or to the end of the sequence if the tile holds a sink key.
__host__ __device__ inline void bwd_key_tile_rows(const BwdParams &p, int kt, int &yt_lo, int &yt_hi)
{
    const int64_t j0 = (int64_t)kt * 64;
    const int64_t j1 = j0 + 63 < p.S ? j0 + 63 : p.S - 1;
    int64_t i_hi = p.S - 1;
    if (j0 >= p.n_sink) {
        const int64_t last = (j1 / p.block + p.window) * p.block - 1;  // window <= S: no overflow
        if (last < i_hi) i_hi = last;
    }
    yt_lo = (int)((j0 * p.G) / 32);
    yt_hi = (int)(((i_hi + 1) * p.G - 1) / 32);
}

bool bwd_group_supported(int G);
hipError_t launch_backward_bf16(const BwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream);

struct F32Params {
    const float *q, *k, *v;
    float *out, *lse;
    int B, Hq, Hkv;
    int64_t S;
    int d_qk, d_v;
    int64_t k_row, v_row;  // elements per key / value row (v_row = d_qk when v aliases k)
    int n_sink, window, block;  // as in FwdParams
    float scale;
    // decode form: one query per sequence at position seqlens[b] - 1 of its cache (k, v are then
    // [B, S, Hkv, .] caches, q and out [B, Hq, .], lse [B, Hq]); nullptr: prefill
    const int32_t *seqlens;
};
hipError_t launch_prefill_f32(const F32Params &p, hipStream_t stream);

// fp32 backward: the forward's tensors plus the stored out and lse, the incoming gradient and the
// three results (dv == nullptr: the values are a prefix of the key rows, dk holds the whole gradient)
struct F32BwdParams {
    const float *q, *k, *v, *out, *lse, *dout;
    float *dq, *dk, *dv;
    int B, Hq, Hkv;
    int64_t S;
    int d_qk, d_v;
    int64_t k_row, v_row;
    int n_sink, window, block;
    float scale;
};
hipError_t launch_backward_f32(const F32BwdParams &p, hipStream_t stream);

}  // namespace loza
#endif
