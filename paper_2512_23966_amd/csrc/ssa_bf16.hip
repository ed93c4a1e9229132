// bf16 streaming-sparse-attention kernels for gfx950 (MI355X): prefill, extend and split-key decode.
//
// What is computed: O* = softmax(scale * Q K*^T) V* over the live key set of every query
// (paper: Architecture section, Eq. 2 / Eq. 4; with a window that covers everything this is Eq. 1),
// plus the natural log of the softmax denominator. The live set of query i is
//   { j <= i : j < n_sink  or  j >= max(0, i / block - window + 1) * block },
// which is the paper's block-granular pattern (sink blocks, local blocks, block size) and, with
// block = 1, the token-granular one (the `window` most recent keys, the query's own included).
// Three forms share one kernel template: prefill (queries = keys = S positions), extend (the q_len
// newest positions of every sequence against its cache, lengths on the device) and decode (one
// query per sequence, the live keys split over several workgroups and merged by a second kernel);
// extend and decode can read a paged cache through a block table.
//
// How it is mapped to the machine (one workgroup = 4 wavefronts = 1 per SIMD; prefill tiles hold
// 128 query rows and all four waves score and accumulate, decode tiles hold 64 rows (the heads of one
// token) and two waves score while the other two accumulate values and issue most tile copies):
//   * Rows of a workgroup tile are (position, head-in-group) pairs of ONE key/value head, so all
//     query heads that share a latent (absorbed MLA) reuse each key tile from a single LDS copy.
//   * Only live key tiles are enumerated: the sink tiles, then the window tiles, by closed-form
//     integer arithmetic (no schedule metadata in memory, the same schedule for every head).
//     Interior tiles take no mask; only tiles cut by the causal diagonal, the window's trailing
//     edge or the sink edge evaluate the predicate per element.
//   * Score phase: a scoring wave holds the 32 query rows of its row block in registers as MFMA B
//     operands and computes S^T = K Q^T for the 32 keys of the tile (32x32x16 bf16 MFMA), so that
//     one lane owns one query row and the online-softmax statistics need a single cross-lane step.
//   * P is rounded to bf16 and handed over through LDS; in the value phase wave w owns the
//     d_v / 4 output columns [w*d_v/4, (w+1)*d_v/4) of ALL rows of the tile, so each value
//     fragment (read transposed from the key tile with ds_read_b64_tr_b16) is fetched once per
//     workgroup instead of once per wave.
//   * Key tiles stream HBM/L2 -> LDS with global_load_lds_dwordx4 (no register staging) through a
//     ring of 3 (prefill) or 4 (decode: more bytes in flight per compute unit) stages; LDS rows
//     are padded by 16 bytes so 128-bit fragment reads are bank-conflict free.
//   * One barrier per tile: while the value phase of tile u runs on the matrix cores, the scores
//     of tile u + 1 are already in registers and their softmax is issued between the matrix
//     instructions; later tiles are in flight from global memory.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "score_asm.h"
#include "ssa_device.h"
#include "ssa_kernels.h"

namespace loza {

// RB: 32-row blocks per workgroup tile. Four wavefronts, one per SIMD.
//   Prefill (RB = 4): every wave scores one row block and accumulates d_v / 4 output columns of
//   all 128 rows.
//   Decode (RB = 2; the 64 rows are the heads of one token): the waves specialise. Waves 0 and 1
//   keep the queries in registers, score and run the softmax; waves 2 and 3 keep the output
//   accumulators (d_v / 2 columns of all rows each) and run the value phase. Neither role needs
//   the other's registers, so both fit, and the two phases of consecutive tiles overlap on
//   different SIMDs.
template <int DQK, int DV, int RB, bool ALIAS, bool DECODE>
struct TileCfg {
    static constexpr int M = 32 * RB;            // query rows per workgroup
    static constexpr int N = 32;                 // keys per tile
    static constexpr int NW = 4;                 // wavefronts
    static constexpr bool SPEC = DECODE;         // specialised roles
    static_assert(SPEC ? RB == 2 : RB == 4, "row blocks per tile");
    static constexpr int VW = SPEC ? 2 : 4;      // waves that accumulate values
    static constexpr int DVW = DV / VW;          // output columns owned by one of them
    static constexpr int DVB = DVW / 32;         // 32-column blocks of them
    static_assert(DVB * 32 * VW == DV, "d_v must be a multiple of 128");
    static_assert(DQK % 16 == 0, "d_qk must be a multiple of 16");
    static constexpr int KROW = DQK * 2 + 16;    // LDS bytes per key row (16 bytes of padding)
    static constexpr int VROW = ALIAS ? KROW : DV * 2 + 16;
    static constexpr int KCPR = KROW / 16;       // 16-byte chunks per padded key row
    static constexpr int VCPR = VROW / 16;
    // global -> LDS copy: one instruction moves 64 consecutive 16-byte chunks (1 KB) of the padded
    // tile. Prefill: instruction i belongs to wave i % 4. Decode: the scoring waves pace the loop and
    // the value waves have time to spare, so the value waves take most copies (between their matrix
    // instructions): the first 2 SC key instructions alternate between the two scoring waves (SC
    // each, woven into their score phase; wide aliased rows only), the rest alternates between the
    // two value waves.
    static constexpr int NCW = SPEC ? VW : NW;   // waves a run of instructions alternates between
    static constexpr int K_INSTR = (N * KCPR + 63) / 64;
    static constexpr int V_INSTR = ALIAS ? 0 : (N * VCPR + 63) / 64;
    static constexpr int SC = (SPEC && DQK == 576 && ALIAS) ? LOZA_SCORE_COPIES_576_W2 : 0;
    static constexpr int K_PER_WAVE = (K_INSTR - 2 * SC + NCW - 1) / NCW;   // of a value wave in decode; SC <= this
    static constexpr int V_PER_WAVE = (V_INSTR + NCW - 1) / NCW;
    static_assert(SC <= K_PER_WAVE, "the copy offsets of a scoring wave share the array of a value wave");
    static constexpr int KTILE = K_INSTR * 1024;
    static constexpr int VTILE = V_INSTR * 1024;
    static constexpr int STAGE = KTILE + VTILE;
    // Ring of tile stages: tile u feeds the value phase, u + 1 the score phase, the rest is in
    // flight. Decode is bound by HBM latency x bandwidth, so it keeps one more tile in flight.
    static constexpr int NSTAGE = DECODE ? 4 : 3;
    // copy instructions one wave issues per tile, at least (waves differ by at most one)
    static constexpr int MIN_COPIES = (K_INSTR - 2 * SC) / NCW + V_INSTR / NCW;
    // Two buffers for P. Rounded to bf16 once, the P of consecutive tiles alternate between them
    // (the softmax of tile u + 1 writes one while the value phase of tile u reads the other). A
    // two-term pass (p = hi + lo, both bf16) keeps hi in the first and lo in the second and pays for
    // the missing double buffer with a second barrier per tile.
    static constexpr int NPBUF = 2;
    static constexpr int PLO = 1;                // index offset of the low-term buffer
    static constexpr int PROW = N * 2 + 16;      // LDS bytes per row of P (padded)
    static constexpr int PBYTES = M * PROW;
    static constexpr int OFF_P = NSTAGE * STAGE;
    static constexpr int OFF_ALPHA = OFF_P + NPBUF * PBYTES;      // float[2][M]
    static constexpr int OFF_FLAG = OFF_ALPHA + 2 * M * 4;        // int[2][4] (one per row block, padded)
    static constexpr int OFF_LPART = OFF_FLAG + 2 * 16;           // float[2][M]
    static constexpr int OFF_REDO = OFF_LPART + 2 * M * 4;        // int: the tile has to be computed again, with two-term P
    static constexpr int LDS_BYTES = OFF_REDO + 16;
    // The softmax between the matrix instructions of the value phase takes the speculative form (below)
    // where that phase has a matrix instruction for every one of its jobs; with fewer (narrow values)
    // the vector ALU is the bound either way and the ordinary form has fewer instructions.
    static constexpr int SPEC_JOBS = 30;
    static constexpr bool SPEC_SOFTMAX = !DECODE && (N / 16) * DVB * RB >= SPEC_JOBS;
    static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit the 160 KB LDS");
};

// One pass over one workgroup tile. PRECISE: P goes to the value phase as two bf16 terms. Returns
// true (the same in every wave) when the tile has been left unwritten for a PRECISE pass.
template <int DQK, int DV, int RB, bool ALIAS, bool DECODE, bool PRECISE, bool OUTF32, bool EXT>
static __device__ __forceinline__ bool ssa_fwd_tile(const FwdParams &p, char *smem)
{
    using C = TileCfg<DQK, DV, RB, ALIAS, DECODE>;
    constexpr int M = C::M, N = C::N, NSTAGE = C::NSTAGE;
    constexpr bool ROTATE = !DECODE;  // prefill and extend walk their window tiles in rotated order (below)

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, lh = lane >> 5;
    constexpr int NW = C::NW;
    constexpr bool SPEC = C::SPEC;
    const bool scorer = !SPEC || wave < RB;   // this wave scores row block `wr` and runs its softmax
    const int wr = scorer ? wave : 0;
    const int vw = SPEC ? wave - RB : wave;   // which slice of the output columns this wave accumulates
    constexpr int NCW = C::NCW;
    const int cw = SPEC ? (scorer ? wave : vw) : wave;               // index within the waves it alternates with
    const int k_first = (SPEC && !scorer) ? 2 * C::SC : 0;             // first key instruction of that run
    const int k_count_max = (SPEC && scorer) ? C::SC : C::K_PER_WAVE;  // key instructions of this wave, at most
    const bool copies_values = !SPEC || !scorer;

    // ---- which tile of which (batch, kv head) ------------------------------------------------
    int id = blockIdx.x;
    if (!DECODE && DQK == 128) {
        // Workgroups go to the eight XCDs round-robin and every XCD has an L2 of its own. With one
        // head per kv group a row tile is 128 positions, and 32 concurrent workgroups that are every
        // eighth row tile make each L2 hold the keys of 32768 positions; handing every XCD one
        // contiguous eighth of the tiles makes them consecutive row tiles (4096 positions).
        // (Measured: a few per cent at 32K tokens. The wide shape, two positions per tile, loses.)
        const int total = gridDim.x, chunk = total / 8;
        if (id < chunk * 8) id = (id % 8) * chunk + id / 8;
    }
    int split = 0;
    if (DECODE) { split = id % p.n_splits; id /= p.n_splits; }
    const int rt = p.rt_begin + p.row_tiles - 1 - (id % p.row_tiles);  // heaviest (latest) row tiles first
    id /= p.row_tiles;
    const int g = id % p.Hkv;
    const int b = id / p.Hkv;
    const int G = p.G;

    // "Extend" prefill: the last q_len positions of each sequence are the queries, the keys come
    // from a cache whose valid length is seqlens[b] (q_len = 0: plain prefill, queries = keys = S).
    constexpr bool extend = EXT;  // (its own instantiation: the plain prefill pays nothing for it)
    // valid key rows (a length beyond the cache is cut to the cache)
    const int64_t L = (DECODE || extend) ? ((int64_t)p.seqlens[b] < p.S ? (int64_t)p.seqlens[b] : p.S) : p.S;
    const int64_t Sq = extend ? (int64_t)p.q_len : p.S;           // query positions per sequence
    const int64_t pos0 = extend ? L - Sq : 0;                     // position of the first of them
    const int64_t R = DECODE ? (int64_t)G : Sq * (int64_t)G;      // query rows of this (b, g)
    const int64_t r0 = (int64_t)rt * M;
    const int n_sink = p.n_sink;
    const int window = p.window, block = p.block;
    auto window_begin = [&](int i) { return window_begin_of(i, window, block); };

    // ---- decode queries with a handful of live keys (or none) belong to the merge kernel ------
    if (DECODE) {
        const int64_t se = n_sink < L ? n_sink : L;
        const int64_t wb = L > 0 ? window_begin_of((int)(L - 1), p.window, p.block) : 0;
        const int64_t n_live = se + (L - (wb > se ? wb : se));
        if (n_live < kDirectKeys) return false;
    }

    // ---- the query row this lane scores ---------------------------------------------------------
    const int64_t my_row = r0 + wr * 32 + ln;
    const int64_t my_row_c = my_row < R ? my_row : R - 1;
    const int r_row = DECODE ? 0 : (int)(my_row_c / G);           // index of the query among the Sq
    const int i_row = DECODE ? (int)(L - 1) : (int)(pos0 + r_row);
    const int i_min = DECODE ? (int)(L - 1) : (int)(pos0 + r0 / G);
    const int i_max = DECODE ? (int)(L - 1) : (int)(pos0 + ((r0 + M - 1 < R) ? r0 + M - 1 : R - 1) / G);
    // Tiles among the first positions, and every tile of a pattern that leaves all rows few live keys,
    // take the two-term pass right away.
    if (!DECODE && !PRECISE && (p.all_precise || i_min < kPrecisePositions)) return true;

    bf16x8 qf[DQK / 16];

    // ---- live key tiles: sink tiles [0, nA), then window tiles [wt0, wt0 + nB) -------------------
    const int sink_end = i_max < 0 ? 0 : (n_sink < i_max + 1 ? n_sink : i_max + 1);
    const int win_begin = window_begin(i_min < 0 ? 0 : i_min);
    const int w_lo_row = window_begin(i_row), w_lo_max = window_begin(i_max);
    int nA = (sink_end + N - 1) / N;
    const int wt0 = win_begin / N, wt1 = i_max / N;
    int nB;
    if (wt0 <= nA) { nA = wt1 + 1; nB = 0; } else { nB = wt1 - wt0 + 1; }
    if (i_max < 0) { nA = 0; nB = 0; }  // queries before the start of the sequence see nothing
    const int n_tiles = nA + nB;
    int t_begin = 0, t_end = n_tiles;
    // A decode split takes every n_splits-th live tile: the splits of a sequence then walk through
    // the same stretch of the cache together (measured a little faster than a contiguous quarter each).
    int t_stride = 1, t_first = 0;
    if (DECODE) {
        t_stride = p.n_splits; t_first = split;
        t_end = n_tiles > split ? (n_tiles - split + p.n_splits - 1) / p.n_splits : 0;
    }
    // Prefill: the window tiles are walked in rotated order, starting at the tile whose index is a
    // multiple of the window's tile count (the softmax does not care about the order). Workgroups that
    // run at the same time on one XCD are neighbouring row tiles whose windows are shifted against each
    // other by a few key tiles; walking each window from its own first tile, they would ask for the
    // same key tile a few steps apart, each of them at another place of its window, and together they
    // would keep a band of keys alive that the XCD's L2 cannot hold (measured at 32K tokens, d = 128:
    // L2 hit rate 25 %, 19 GB fetched for 0.5 GB of keys and values). Rotated, every one of them asks
    // for the key tile t (mod the window's tile count) at its step t, and one fetch into L2 serves them
    // all (hit rate 85 %, 3.7 GB).
    int w_rot = 0;
    if (ROTATE && nB > 1) { w_rot = wt0 % nB; w_rot = w_rot == 0 ? 0 : nB - w_rot; }
    auto key_tile = [&](int t) {
        const int tt = t_first + t * t_stride;
        if (tt < nA) return tt;
        int x = tt - nA;
        if (ROTATE) { x += w_rot; x = x >= nB ? x - nB : x; }
        return wt0 + x;
    };

    // ---- global -> LDS copy plan (the same for every tile) --------------------------------------
    // Copy instruction `instr` fills LDS slots [instr*64, instr*64 + 64) of the padded tile: slot p
    // is chunk p % cpr of row p / cpr. Within one instruction the row changes at most once, at lane
    // `lb` when a row has at least 64 chunks; lanes below it take byte offset offA + 16*lane into
    // the global tile, the others offB + 16*lane. A padding slot fetches the chunk that follows its
    // row in memory and slots past the tile fetch further on; both are cut to the last valid chunk
    // below and never read back from LDS.
    const uint32_t pos_stride_k = (uint32_t)p.Hkv * DQK * 2;  // bytes between consecutive positions
    const uint32_t pos_stride_v = (uint32_t)p.Hkv * DV * 2;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    auto copy_offset = [&](int instr, int cpr, uint32_t stride) {
        const int p0 = instr * 64, row0 = p0 / cpr, c0 = p0 - row0 * cpr;
        if (cpr >= 64) {
            const int lb = cpr - c0;  // first lane of the next row (>= 64: no row change inside)
            const uint32_t offA = (uint32_t)row0 * stride + (uint32_t)c0 * 16u;
            const uint32_t offB = (uint32_t)(row0 + 1) * stride - (uint32_t)lb * 16u;
            return (lane < lb ? offA : offB) + lane16;
        }
        const int pl = p0 + lane, row = pl / cpr;
        return (uint32_t)row * stride + (uint32_t)(pl - row * cpr) * 16u;
    };
    uint32_t kvoff[C::K_PER_WAVE];
#pragma unroll
    for (int u = 0; u < C::K_PER_WAVE; ++u) kvoff[u] = copy_offset(k_first + u * NCW + cw, C::KCPR, pos_stride_k);
    uint32_t vvoff[C::V_PER_WAVE > 0 ? C::V_PER_WAVE : 1];
#pragma unroll
    for (int u = 0; u < C::V_PER_WAVE; ++u) vvoff[u] = copy_offset(u * NCW + cw, C::VCPR, pos_stride_v);

    const uint32_t smem_lds = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)smem);
    // A paged cache (decode only) keeps the rows of a sequence in pages of 2^page_shift rows that a
    // block table maps to physical pages; a key tile never straddles a page (pages hold a multiple
    // of N rows), so paging only changes where a tile starts.
    const bool paged = (DECODE || EXT) && p.block_table != nullptr;  // a plain prefill has no table
    const int64_t seq_row0 = paged ? 0 : (int64_t)b * p.S;
    const char *kbase = (const char *)p.k + (seq_row0 * p.Hkv + g) * (int64_t)DQK * 2;
    const char *vbase = (const char *)p.v + (seq_row0 * p.Hkv + g) * (int64_t)DV * 2;
    // The block-table entry of key tile t is fetched by a scalar buffer load: it must not count as a
    // vector load (the tile loop waits on exact counts of those), and it has to be a load the compiler
    // knows about, so that the compiler places the wait before the first use of the value, however it
    // moves the value between registers meanwhile. (A load spelled out in an asm statement, with the
    // wait in a second statement, is not safe: the register may be copied between the two, before the
    // data is there.) The tile loop asks for the entry one iteration ahead, so the latency is hidden.
    // The buffer is this sequence's row of the table; an offset beyond it reads 0.
    const i32x4 table_rsrc = paged ? table_row_resource(p.block_table + (int64_t)b * p.max_pages, p.max_pages) : i32x4{0, 0, 0, 0};
    auto page_request = [&](int t) -> int32_t {
        if (!paged) return 0;
        const int64_t j0 = (int64_t)key_tile(t) * N;
        return llvm_amdgcn_s_buffer_load_i32(table_rsrc, (int32_t)((uint32_t)(j0 >> p.page_shift) * 4u), 0);
    };
    auto page_wait = [&](int32_t pid) -> int32_t { return pid; };
    // cache row (relative to kbase / vbase) at which key tile t starts, given its block-table entry
    auto tile_row = [&](int t, int32_t pid) -> int64_t {
        const int64_t j0 = (int64_t)key_tile(t) * N;
        if (paged) {
            pid = pid < 0 ? 0 : (pid < p.num_pages ? pid : p.num_pages - 1);  // a bad entry stays in bounds
            return ((int64_t)pid << p.page_shift) + (j0 & ((1 << p.page_shift) - 1));
        }
        return j0;
    };

    // One global -> LDS copy instruction: 64 lanes x 16 bytes from base + off (per lane) to the 1 KB
    // of LDS at lds_addr (wave-uniform, through M0). Spelled out in asm so that the compiler's
    // wait-count bookkeeping does not know about it: it would otherwise drain every copy in flight
    // (vmcnt(0)) before the next LDS read, and the tile loop waits with explicit counts instead.
    // A decode reads every cache row once: its copies carry the non-temporal hint (measured on this
    // access pattern: 6.9 TB/s against 6.0 TB/s without). A prefill reads its keys again and again
    // from L2 and keeps the default policy.
    auto copy_1k = [&](const char *base, uint32_t off, uint32_t lds_addr) {
        if constexpr (DECODE)
            asm volatile("s_mov_b32 m0, %2\n s_nop 0\n global_load_lds_dwordx4 %0, %1 nt"
                         :: "v"(off), "s"(base), "s"(lds_addr) : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %2\n s_nop 0\n global_load_lds_dwordx4 %0, %1"
                         :: "v"(off), "s"(base), "s"(lds_addr) : "memory", "m0");
    };
    // what the copy instructions of one key tile share (wave-uniform): the tile starts at cache row `row`
    struct TileCopy {
        const char *ksrc, *vsrc;
        uint32_t kdst, vdst, kmax, vmax;
    };
    // byte offset of cache row `row` (a row index fits 32 bits unless the cache is paged)
    auto tile_bytes = [&](int64_t row, uint32_t stride) -> int64_t {
        return paged ? row * (int64_t)stride : (int64_t)((uint64_t)(uint32_t)row * stride);
    };
    auto plan_copy = [&](int t, int stage, int64_t row) {
        // rows of the tile at or past the sequence end fetch from its last valid row instead:
        // they are dead (j > i) and only have to be finite
        const int left = (int)L - 1 - key_tile(t) * N;
        const uint32_t lim = left < N - 1 ? (uint32_t)left : (uint32_t)(N - 1);
        TileCopy tc;
        tc.ksrc = kbase + tile_bytes(row, pos_stride_k);
        tc.kdst = smem_lds + stage * C::STAGE + (k_first + cw) * 1024;
        tc.kmax = lim * pos_stride_k + (C::KCPR - 2) * 16;
        tc.vsrc = vbase + tile_bytes(row, pos_stride_v);
        tc.vdst = smem_lds + stage * C::STAGE + C::KTILE + cw * 1024;
        tc.vmax = lim * pos_stride_v + (C::VCPR - 2) * 16;
        return tc;
    };
    // copy instruction c of this wave: its key copies first, then (separate values) its value copies
    constexpr int COPIES_PER_WAVE = C::K_PER_WAVE + C::V_PER_WAVE;
    auto copy_nth = [&](const TileCopy &tc, int c) {
        if (c < C::K_PER_WAVE) {
            const int u = c;
            if (u < k_count_max && k_first + u * NCW + cw < C::K_INSTR)  // wave-uniform
                copy_1k(tc.ksrc, kvoff[u] < tc.kmax ? kvoff[u] : tc.kmax, tc.kdst + u * (NCW * 1024));
        } else if (!ALIAS) {
            const int u = c - C::K_PER_WAVE;
            if (copies_values && u * NCW + cw < C::V_INSTR)
                copy_1k(tc.vsrc, vvoff[u] < tc.vmax ? vvoff[u] : tc.vmax, tc.vdst + u * (NCW * 1024));
        }
    };
    // this wave's copy instructions [c_first, ...) of key tile t into `stage`
    auto issue_tile = [&](int t, int stage, int c_first, int64_t row) {
        const TileCopy tc = plan_copy(t, stage, row);
#pragma unroll
        for (int c = 0; c < COPIES_PER_WAVE; ++c)
            if (c >= c_first) copy_nth(tc, c);
    };

    f32x16 o[C::DVB][RB];
#pragma unroll
    for (int db = 0; db < C::DVB; ++db)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][rb][e] = 0.f;
    float m_ref = LOZA_NEG_INF;  // reference maximum of scale*log2(e)*q.k the exponentials are taken against
    // This lane's share of the running row sums: of the exponentials as computed (-> log-sum-exp)
    // and of the same values after rounding to bf16 (-> the normaliser of O, which is accumulated
    // from the rounded values: the weights then sum to one exactly).
    float l_run = 0.f, lr_run = 0.f;

    float *s_alpha = (float *)(smem + C::OFF_ALPHA);
    int *s_flag = (int *)(smem + C::OFF_FLAG);
    float *s_lpart = (float *)(smem + C::OFF_LPART);
    char *s_p = smem + C::OFF_P;
    int *s_redo = (int *)(smem + C::OFF_REDO);
    if (tid < 8) s_flag[tid] = 0;  // the padding entries of the flag words never ask for a rescale
    if (!PRECISE && tid == 8) *s_redo = 0;

    // ---- scores of one tile: S^T[32 keys][32 rows of block wr] ------------------------------------
    // One inline-asm statement (score_asm.h): key fragment kk + DEPTH is fetched from LDS while
    // fragment kk feeds the matrix core, with the exact lgkmcnt each step needs. The accumulator is
    // in VGPRs (the AGPR half of the register file is full of O).
    constexpr bool WEAVE = (DQK == 576 && ALIAS);  // copy instructions woven into the score phase
    // The same with the copy of key tile `t_copy` into stage `stage_copy` woven in (wide rows only):
    // the copy instructions issue between matrix instructions instead of ahead of them.
    auto score_tile_copy = [&](int stage, f32x16 &s, int t_copy, int stage_copy, int64_t row_copy) {
        if constexpr (WEAVE) {
            const uint32_t kaddr = smem_lds + stage * C::STAGE + ln * C::KROW + lh * 16;
            // (scalar arithmetic the wave has nothing to overlap with: 32-bit where the values allow)
            const int left = (int)L - 1 - key_tile(t_copy) * N;  // rows of the tile after its first that exist
            const uint32_t lim = left < N - 1 ? (uint32_t)left : (uint32_t)(N - 1);
            const char *ksrc = kbase + tile_bytes(row_copy, pos_stride_k);
            const uint32_t kmax = lim * pos_stride_k + (C::KCPR - 2) * 16;
            const uint32_t m0base = smem_lds + stage_copy * C::STAGE + wave * 1024;
            static_assert(!WEAVE || DECODE || (LOZA_SCORE_COPIES_576_W4 * NW <= C::K_INSTR && C::K_PER_WAVE <= LOZA_SCORE_COPIES_576_W4 + 1), "copy plan");
            bf16x8 kf[LOZA_SCORE_DEPTH_576];
            uint32_t tmp;
            // prefill: 9 of this wave's 9 or 10 copies, every fourth instruction of the tile; decode: the
            // 4 copies of a scoring wave, every second of the first eight, marked as read-once
            if constexpr (DECODE) LOZA_SCORE_PHASE_576_COPY_W2_NT(s, kf, tmp, kaddr, qf, kvoff, kmax, ksrc, m0base);
            else LOZA_SCORE_PHASE_576_COPY_W4(s, kf, tmp, kaddr, qf, kvoff, kmax, ksrc, m0base);
        }
    };
    auto score_tile = [&](int stage, f32x16 &s) {
        const uint32_t kaddr = smem_lds + stage * C::STAGE + ln * C::KROW + lh * 16;
        static_assert(DQK == 576 || DQK == 128, "add a LOZA_SCORE_PHASE for this d_qk");
        if constexpr (DQK == 576) {
            bf16x8 kf[LOZA_SCORE_DEPTH_576];
            LOZA_SCORE_PHASE_576(s, kf, kaddr, qf);
        } else {
            bf16x8 kf[LOZA_SCORE_DEPTH_128];
            LOZA_SCORE_PHASE_128(s, kf, kaddr, qf);
        }
    };

    // ---- mask + online softmax of one tile; P (bf16), alpha and the rescale flag go to LDS ----------
    float sm_m_use = 0.f, sm_alpha = 1.f, sm_psum = 0.f, sm_rsum = 0.f, sm_mx = 0.f;
    bool sm_up = false;
    uint32_t sm_pk[8];
    uint32_t sm_pk_lo[PRECISE ? 8 : 1];
    auto sm_mask = [&](f32x16 &s, const int j0) {
        // tiles the pattern cuts: causal diagonal, trailing edge of the window, end of the sink
        // (j0 + N - 1 cannot overflow: j0 <= 0x3fffffff, the "no such tile" marker, masks everything)
        const bool interior = (j0 + N - 1 <= i_min) && ((j0 + N - 1 < n_sink) || (j0 >= w_lo_max));
        if (!interior) {
            const int jb = j0 + 4 * lh;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int j = jb + 8 * (e >> 2) + (e & 3);
                const bool ok = (j <= i_row) & ((j < n_sink) | (j >= w_lo_row));
                s[e] = ok ? s[e] : LOZA_NEG_INF;
            }
        }
    };
    auto sm_max8 = [&](const f32x16 &s, const int e0) {
        float mx = s[e0];
#pragma unroll
        for (int e = e0 + 1; e < e0 + 8; ++e) mx = fmaxf(mx, s[e]);
        return mx;
    };
    auto sm_decide = [&](float mx, const float lazy) {
        sm_up = mx > m_ref + lazy;  // also true on the first live tile (m_ref = -inf)
        const float m_new = sm_up ? mx : m_ref;
        sm_alpha = sm_up ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.0f;
        m_ref = m_new;
        sm_m_use = (m_new == LOZA_NEG_INF) ? 0.f : m_new;  // row with no live key so far
        sm_psum = 0.f;
        sm_rsum = 0.f;
    };
    auto sm_end_fn = [&](const int pbuf) {
        l_run = l_run * sm_alpha + sm_psum;
        lr_run = lr_run * sm_alpha + sm_rsum;
        const bool rescale = __any(sm_up);
        if (lane == 0) s_flag[pbuf * 4 + wr] = rescale ? 1 : 0;
        if (rescale && lh == 0) s_alpha[pbuf * M + wr * 32 + ln] = sm_alpha;
        char *pp = s_p + (PRECISE ? 0 : pbuf) * C::PBYTES + (wr * 32 + ln) * C::PROW + (4 * lh) * 2;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            u32x2 w;
            w[0] = sm_pk[2 * qd];
            w[1] = sm_pk[2 * qd + 1];
            *(u32x2 *)(pp + qd * 16) = w;
            if (PRECISE) {
                w[0] = sm_pk_lo[2 * qd];
                w[1] = sm_pk_lo[2 * qd + 1];
                *(u32x2 *)(pp + C::PLO * C::PBYTES + qd * 16) = w;
            }
        }
    };
    // The softmax as a list of micro-jobs, one or a few of which are issued after each matrix
    // instruction of the value phase: 0 mask + maximum of scores 0..7, 1 maximum of 8..15, 2 other
    // wavefront half + scale, 3 reference update, then per pair of scores i: 4+3i and 5+3i one
    // exponential each, 6+3i bf16 pack + running sums; last the hand-over through LDS. The empty asm
    // statements anchor each job's results in its slot (the optimiser otherwise sinks all of this
    // arithmetic below the last matrix instruction); where the softmax runs on its own (the decode's
    // scoring waves) there are none, and the sixteen independent chains overlap as the scheduler likes.
    constexpr int SM_JOBS = 4 + 3 * 8 + 1;
    auto sm_job = [&](auto anchored, const int j, f32x16 &s, const int j0, const float lazy, const int pbuf) {
        constexpr bool ANCHOR = decltype(anchored)::value;
        const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
        if (j == 0) {
            sm_mask(s, j0);
            sm_mx = sm_max8(s, 0);
            if constexpr (ANCHOR) asm volatile("" : "+v"(s), "+v"(sm_mx));
        } else if (j == 1) {
            sm_mx = fmaxf(sm_mx, sm_max8(s, 8));
            if constexpr (ANCHOR) asm volatile("" : "+v"(sm_mx));
        } else if (j == 2) {
            sm_mx = max_with_other_half(sm_mx) * p.scale_log2;  // scale > 0: maximum of the scaled scores
            if constexpr (ANCHOR) asm volatile("" : "+v"(sm_mx));
        } else if (j == 3) {
            sm_decide(sm_mx, lazy);
            if constexpr (ANCHOR) asm volatile("" : "+v"(sm_alpha), "+v"(sm_m_use), "+v"(m_ref));
        } else if (j < SM_JOBS - 1) {
            const int i = (j - 4) / 3, part = (j - 4) % 3, e = 2 * i;
            if (part == 0) {
                // exp2(scale*log2(e)*s - m): a dead key (s = -inf) gives exactly 0
                s[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], p.scale_log2, -sm_m_use));
                if constexpr (ANCHOR) asm volatile("" : "+v"(s));
            } else if (part == 1) {
                s[e + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e + 1], p.scale_log2, -sm_m_use));
                if constexpr (ANCHOR) asm volatile("" : "+v"(s));
            } else {
                sm_pk[i] = pack_bf16(s[e], s[e + 1]);
                if (PRECISE) {
                    // second bf16 term of each weight: what the first rounding lost
                    const float h0 = __builtin_bit_cast(float, sm_pk[i] << 16), h1 = __builtin_bit_cast(float, sm_pk[i] & 0xffff0000u);
                    sm_pk_lo[i] = pack_bf16(s[e] - h0, s[e + 1] - h1);
                    if constexpr (ANCHOR) asm volatile("" : "+v"(sm_pk_lo[i]));
                }
                sm_psum += s[e] + s[e + 1];
                // the sum of the two rounded values, by one dot product with (1, 1)
                sm_rsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, sm_pk[i]), ones, sm_rsum, false);
                if (PRECISE) sm_rsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, sm_pk_lo[i]), ones, sm_rsum, false);
                if constexpr (ANCHOR) asm volatile("" : "+v"(sm_psum), "+v"(sm_rsum), "+v"(sm_pk[i]));
            }
        } else if (j == SM_JOBS - 1) {
            sm_end_fn(pbuf);
        }
    };
    auto softmax_tile = [&](f32x16 &s, const int j0, const int pbuf, const float lazy) {
#pragma unroll
        for (int j = 0; j < SM_JOBS; ++j) sm_job(std::false_type{}, j, s, j0, lazy, pbuf);
    };
    // The same softmax for the value phase of prefill and extend, where the reference almost never
    // moves: the exponentials are taken against the CURRENT reference at once, without waiting for the
    // tile's maximum (a serial chain of some thirty instructions through a cross-lane exchange), and
    // the largest weight is checked afterwards. Measured on gfx950, one wave per SIMD: behind one
    // 32x32x16 matrix instruction (32 cycles) an exponential and three simple vector instructions
    // issue for free if none of them waits for the one before (a dependent instruction issues 8
    // cycles after the one it waits for, an independent one after 4), while a bf16 dot-product
    // instruction holds up the matrix pipeline for 16 cycles. So every job below is a handful of
    // instructions that depend on EARLIER jobs only (element e + 1 is scaled while element e - 1 is
    // exponentiated and the pair before is packed and summed), and the sum of the rounded weights is
    // taken with shifts and adds. If a weight exceeds the threshold (2^lazy; 2^0 in an exact tile) or a
    // row has no reference yet, the wave says so (sm_bad, uniform) and the caller takes the tile's scores
    // again and runs the ordinary softmax: the result is the one the ordinary order gives.
    constexpr int SPEC_JOBS = C::SPEC_JOBS;
    bool sm_bad = false;
    float sm_pm = 0.f, sm_ra = 0.f, sm_rb = 0.f, sm_lo = 0.f, sm_hi = 0.f;
    auto sm_job_spec = [&](const int j, f32x16 &s, const int j0, const float thresh, const int pbuf) {
        auto F = [&](int e) { s[e] = __builtin_fmaf(s[e], p.scale_log2, -sm_m_use); };
        auto E = [&](int e) { s[e] = __builtin_amdgcn_exp2f(s[e]); };
        if (j == 0) {
            sm_mask(s, j0);
            sm_m_use = (m_ref == LOZA_NEG_INF) ? 0.f : m_ref;
            sm_alpha = 1.0f;
            sm_up = false;
            sm_psum = 0.f;
            sm_pm = 0.f;
            sm_ra = 0.f;
            sm_rb = 0.f;
            F(0);
            F(1);
            asm volatile("" : "+v"(s), "+v"(sm_m_use));
        } else if (j <= 18) {
            // one exponential, one scaling, and two instructions of a pair whose exponentials are done
            if (j - 1 < 16) E(j - 1);
            if (j + 1 < 16) F(j + 1);
            if (j >= 3 && (j & 1)) {
                const int i = (j - 3) / 2;
                sm_pk[i] = pack_bf16(s[2 * i], s[2 * i + 1]);
                sm_psum += s[2 * i];
                asm volatile("" : "+v"(sm_pk[i]), "+v"(sm_psum));
            } else if (j >= 4) {
                const int i = (j - 4) / 2;
                sm_psum += s[2 * i + 1];
                sm_pm = fmaxf(fmaxf(sm_pm, s[2 * i]), s[2 * i + 1]);
                asm volatile("" : "+v"(sm_psum), "+v"(sm_pm));
            }
            asm volatile("" : "+v"(s));
        } else if (j == 19) {
            // (not (pm <= thresh): a NaN weight also takes the ordinary path)
            sm_bad = __any(!(sm_pm <= thresh) || m_ref == LOZA_NEG_INF);
        } else if (j <= 28) {
            // the two halves of pair i are widened while those of pair i - 1 are added, on two accumulators
            const int i = j - 20;
            if (i >= 1) {
                sm_ra += sm_lo;
                sm_rb += sm_hi;
            }
            if (i < 8) {
                sm_lo = __builtin_bit_cast(float, sm_pk[i] << 16);
                sm_hi = __builtin_bit_cast(float, sm_pk[i] & 0xffff0000u);
            }
            if (i == 8) sm_rsum = sm_ra + sm_rb;
            asm volatile("" : "+v"(sm_ra), "+v"(sm_rb), "+v"(sm_lo), "+v"(sm_hi), "+v"(sm_rsum));
        } else if (j == 29) {
            if (__builtin_expect(!sm_bad, 1)) sm_end_fn(pbuf);
        }
    };

    // ---- accumulator rescale of one tile (rare after the first tiles) -----------------------------------
    auto rescale_flags = [&](const int pbuf) { return *(const u32x4 *)(s_flag + pbuf * 4); };
    auto rescale_tile = [&](const int pbuf, const u32x4 flags) {
        // one test covers the common case that no row block of the tile moved its reference
        if (__builtin_amdgcn_readfirstlane(flags[0] | flags[1] | flags[2] | flags[3]) == 0) return;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (__builtin_amdgcn_readfirstlane(flags[rb])) {
                const float a = s_alpha[pbuf * M + rb * 32 + ln];
#pragma unroll
                for (int db = 0; db < C::DVB; ++db) {
                    // The accumulators live in the AGPR half of the register file; the empty asm
                    // statements pin them there on both sides of the multiply, so the compiler
                    // moves 16 values through VGPRs at a time instead of evicting the Q fragments.
                    f32x16 t = o[db][rb];
                    asm volatile("" : "+a"(t));
#pragma unroll
                    for (int e = 0; e < 16; ++e) t[e] *= a;
                    asm volatile("" : "+a"(t));
                    o[db][rb] = t;
                }
            }
        }
    };

    // ---- values of one tile: O^T[d_v slice of this wave][all rows] += V^T P^T -------------------------
    // Explicit software pipeline over the (key step, column block) pairs: the value fragments of the
    // pair after next are fetched from LDS while the RB matrix instructions of this pair run. On a
    // scoring wave the softmax of the NEXT tile (scores in `s`) is issued as micro-jobs between the
    // matrix instructions, so that the vector ALUs work in the shadow of the matrix cores.
    struct ValueFrags {
        bf16x8 pf[2][RB];      // P^T fragments of two key steps
        s16x4 vlo[3], vhi[3];  // value fragments: two steps of look-ahead
    };
    constexpr int V_KS = N / 16, V_NSTEP = V_KS * C::DVB;
    auto value_ptrs = [&](const int stage, const int pbuf, const char *&vp, const char *&pb) {
        const char *vtile = smem + stage * C::STAGE + (ALIAS ? 0 : C::KTILE);
        const int s16 = lane & 15, g16 = (lane >> 4) & 1;
        vp = vtile + (lh * 8 + (s16 >> 2)) * C::VROW + (vw * C::DVW + g16 * 16 + (s16 & 3) * 4) * 2;
        pb = s_p + (PRECISE ? 0 : pbuf) * C::PBYTES + ln * C::PROW + lh * 16;
    };
    auto load_v = [&](const char *vp, int step, s16x4 &lo, s16x4 &hi) {
        const char *va = vp + (step / C::DVB) * 16 * C::VROW + (step % C::DVB) * 64;
        lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(va));
        hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(va + 4 * C::VROW));
    };
    // The first fragments of a value phase, requested BEFORE the score phase so that their LDS
    // latency hides behind it.
    auto value_prefetch = [&](const int stage, const int pbuf, ValueFrags &f) {
        const char *vp, *pb;
        value_ptrs(stage, pbuf, vp, pb);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) f.pf[0][rb] = *(const bf16x8 *)(pb + rb * 32 * C::PROW);
        load_v(vp, 0, f.vlo[0], f.vhi[0]);
        if (V_NSTEP > 1) load_v(vp, 1, f.vlo[1], f.vhi[1]);
    };
    auto value_tile = [&](const int stage, const int pbuf, ValueFrags &f, auto with_softmax, f32x16 &s,
                          const int j0_next, const int pbuf_next, const float lazy, auto &&after_slot) {
        constexpr int SM_MODE = decltype(with_softmax)::value;   // 0 none, 1 the job list, 2 the speculative job list
        constexpr bool WITH_SOFTMAX = SM_MODE == 1;
        constexpr int KS = V_KS, NSTEP = V_NSTEP;
        const char *vp, *pb;
        value_ptrs(stage, pbuf, vp, pb);
        const char *pb_lo = pb + C::PLO * C::PBYTES;
        auto &pf = f.pf;
        auto &vlo = f.vlo;
        auto &vhi = f.vhi;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int step = 0; step < NSTEP; ++step) {
            const int ks = step / C::DVB, db = step % C::DVB;
            if (step + 2 < NSTEP) load_v(vp, step + 2, vlo[(step + 2) % 3], vhi[(step + 2) % 3]);
            if (db == 0 && ks + 1 < KS) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) pf[(ks + 1) & 1][rb] = *(const bf16x8 *)(pb + rb * 32 * C::PROW + (ks + 1) * 32);
            }
            s16x8 a8;
            const s16x4 lo = vlo[step % 3], hi = vhi[step % 3];
            a8[0] = lo[0]; a8[1] = lo[1]; a8[2] = lo[2]; a8[3] = lo[3];
            a8[4] = hi[0]; a8[5] = hi[1]; a8[6] = hi[2]; a8[7] = hi[3];
            const bf16x8 a = __builtin_bit_cast(bf16x8, a8);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[ks & 1][rb], o[db][rb], 0, 0, 0);
                if (PRECISE) {
                    const bf16x8 pl = *(const bf16x8 *)(pb_lo + rb * 32 * C::PROW + ks * 32);
                    o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pl, o[db][rb], 0, 0, 0);
                }
                // the micro-jobs of the next tile's softmax that belong to this slot
                constexpr int NSLOT = NSTEP * RB, JPS = (SM_JOBS + NSLOT - 1) / NSLOT;
                const int slot = step * RB + rb;
                if (WITH_SOFTMAX) {
#pragma unroll
                    for (int jj = 0; jj < JPS; ++jj)
                        // (two-term pass: the hand-over, the last job, waits for a barrier of its own)
                        if (slot * JPS + jj < SM_JOBS - (PRECISE ? 1 : 0)) sm_job(std::true_type{}, slot * JPS + jj, s, j0_next, lazy, pbuf_next);
                }
                if (SM_MODE == 2) {
                    constexpr int JPS2 = (SPEC_JOBS + NSLOT - 1) / NSLOT;
#pragma unroll
                    for (int jj = 0; jj < JPS2; ++jj)
                        if (slot * JPS2 + jj < SPEC_JOBS) sm_job_spec(slot * JPS2 + jj, s, j0_next, lazy, pbuf_next);   // (lazy: the threshold 2^lazy)
                }
                after_slot(slot, NSLOT);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // ---- the tile loop: one barrier per tile ------------------------------------------------------------
    // Tile u (ring stage u % NSTAGE) feeds the value phase while the scores of tile u + 1 are taken
    // and tile u + NSTAGE - 1 starts its way from global memory; tiles in between are in flight.
    // Past the last tile the score phase runs on a stale stage and its result is masked out as a
    // whole (key index "infinity"), which leaves the softmax state untouched: one straight-line
    // loop body instead of a peeled last iteration.
    const int nt = t_end - t_begin;
    constexpr int AHEAD = NSTAGE - 1;  // tiles requested ahead of the one in the value phase
    f32x16 s;
    if (nt > 0) {
#pragma unroll
        for (int a = 0; a < AHEAD; ++a)
            if (a < nt) issue_tile(t_begin + a, a, 0, tile_row(t_begin + a, page_wait(page_request(t_begin + a))));
        // The query fragments are requested after the first key tiles, so that both first-touch
        // latencies run together; the score phase waits for them (and with them for every copy
        // issued so far) through the compiler's own wait count.
        if (scorer) {
            const int hh = DECODE ? (int)my_row_c : (int)(my_row_c - (int64_t)r_row * G);
            const int64_t qrow = DECODE ? ((int64_t)b * p.Hq + (int64_t)g * G + hh)
                                        : (((int64_t)b * Sq + r_row) * p.Hq + (int64_t)g * G + hh);
            const uint16_t *qp = p.q + qrow * DQK + lh * 8;
#pragma unroll
            for (int kk = 0; kk < DQK / 16; ++kk) qf[kk] = *(const bf16x8 *)(qp + kk * 16);
        }
        // tile 0 has landed when at most the copies of the later ones are outstanding
        if (nt < AHEAD) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        else if (SPEC && scorer) __builtin_amdgcn_s_waitcnt(vmcnt_imm((AHEAD - 1) * C::SC));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm((AHEAD - 1) * C::MIN_COPIES));
        lds_barrier();
        if (scorer) {
            score_tile(0, s);
            softmax_tile(s, key_tile(t_begin) * N, 0, 0.f);
        }
    }
    auto top_of_tile = [&](int u) {
        // this wave's share of tile u + 1 has landed when at most the copies of the tiles after it
        // are outstanding
        if (u + AHEAD > nt) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        else if (SPEC && scorer) __builtin_amdgcn_s_waitcnt(vmcnt_imm((AHEAD - 2) * C::SC));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm((AHEAD - 2) * C::MIN_COPIES));
        lds_barrier();  // ... everyone's; P of tile u is visible; the stage of tile u - 1 is free
    };
    constexpr int WOVEN = LOZA_SCORE_COPIES_576_W4;
    // where the tile issued in iteration u starts: looked up one iteration ahead (a paged cache
    // reads its block table here, and the answer is there when the copies are issued)
    auto tile_ahead = [&](int u) { return t_begin + u + AHEAD < t_end ? t_begin + u + AHEAD : t_end - 1; };
    int32_t page_pre = nt > 0 ? page_request(tile_ahead(0)) : 0;
    const float lazy_thresh = __builtin_amdgcn_exp2f(p.lazy_log2);
    if (!SPEC) {
        int st_v = 0;  // ring stage of tile u
        for (int u = 0; u < nt; ++u) {
            top_of_tile(u);
            const int64_t row_now = tile_row(tile_ahead(u), page_wait(page_pre));
            page_pre = page_request(tile_ahead(u + 1));
            const int st_k = st_v + 1 < NSTAGE ? st_v + 1 : 0;
            const int st_l = st_v == 0 ? NSTAGE - 1 : st_v - 1;  // = (u + AHEAD) % NSTAGE
            const bool more = u + AHEAD < nt;
            const u32x4 flags = rescale_flags(u & 1);  // requested now, used after the score phase
            ValueFrags vf;
            value_prefetch(st_v, u & 1, vf);
            __builtin_amdgcn_sched_barrier(0);
            if (WEAVE && more) {
                score_tile_copy(st_k, s, t_begin + u + AHEAD, st_l, row_now);
                issue_tile(t_begin + u + AHEAD, st_l, WOVEN, row_now);  // what was not woven in
            } else {
                if (more) issue_tile(t_begin + u + AHEAD, st_l, 0, row_now);
                score_tile(st_k, s);
            }
            rescale_tile(u & 1, flags);
            {
                const int j0_next = u + 1 < nt ? key_tile(t_begin + u + 1) * N : 0x3fffffff;
                const bool exact = u + 1 < p.exact_tiles;
                if constexpr (PRECISE || !C::SPEC_SOFTMAX) {
                    value_tile(st_v, u & 1, vf, std::integral_constant<int, 1>{}, s, j0_next, (u + 1) & 1, exact ? 0.f : p.lazy_log2, [](int, int) {});
                } else {
                    // (one instantiation of the value phase in the loop: with the ordinary and the
                    // speculative form side by side the register allocator spills. An exact tile is a
                    // speculative one with the threshold 2^0.)
                    value_tile(st_v, u & 1, vf, std::integral_constant<int, 2>{}, s, j0_next, (u + 1) & 1, exact ? 1.0f : lazy_thresh, [](int, int) {});
                    if (__builtin_expect(sm_bad, 0)) {
                        // the reference has to move (or the row has none yet): scores again, ordinary softmax
                        score_tile(st_k, s);
                        softmax_tile(s, j0_next, (u + 1) & 1, exact ? 0.f : p.lazy_log2);
                    }
                }
            }
            if constexpr (PRECISE) {
                // every wave has read P of tile u: the single pair of buffers can take P of tile u + 1
                lds_barrier();
                sm_end_fn((u + 1) & 1);
            }
            st_v = st_k;
        }
    } else if (scorer) {
        // scoring role: while the value waves work on tile u, take the scores of tile u + 1 and hand
        // its P over through LDS (score phase and softmax of a tile pace the loop: these waves issue
        // only the few copies that fit between their matrix instructions at no cost)
        int st_v = 0;
        for (int u = 0; u < nt; ++u) {
            top_of_tile(u);
            const int64_t row_now = tile_row(tile_ahead(u), page_wait(page_pre));
            page_pre = page_request(tile_ahead(u + 1));
            const int st_k = st_v + 1 < NSTAGE ? st_v + 1 : 0;
            const int st_l = st_v == 0 ? NSTAGE - 1 : st_v - 1;
            if (WEAVE && u + AHEAD < nt) score_tile_copy(st_k, s, t_begin + u + AHEAD, st_l, row_now);
            else score_tile(st_k, s);
            softmax_tile(s, u + 1 < nt ? key_tile(t_begin + u + 1) * N : 0x3fffffff, (u + 1) & 1,
                         u + 1 < p.exact_tiles ? 0.f : p.lazy_log2);
            st_v = st_k;
        }
    } else {
        // value role
        int st_v = 0;
        for (int u = 0; u < nt; ++u) {
            top_of_tile(u);
            const int64_t row_now = tile_row(tile_ahead(u), page_wait(page_pre));
            page_pre = page_request(tile_ahead(u + 1));
            const int st_l = st_v == 0 ? NSTAGE - 1 : st_v - 1;
            const u32x4 flags = rescale_flags(u & 1);
            ValueFrags vf;
            value_prefetch(st_v, u & 1, vf);
            // the copies of tile u + AHEAD go out between the matrix instructions of this value phase
            // (all at once they fill the memory pipeline's queue and stall the wave)
            const bool more = u + AHEAD < nt;
            const TileCopy tc = plan_copy(more ? t_begin + u + AHEAD : t_begin + u, st_l, row_now);
            rescale_tile(u & 1, flags);
            value_tile(st_v, u & 1, vf, std::integral_constant<int, 0>{}, s, 0, 0, 0.f, [&](int slot, int n_slots) {
                const int per_slot = (COPIES_PER_WAVE + n_slots - 1) / n_slots;
#pragma unroll
                for (int c = slot * per_slot; c < (slot + 1) * per_slot; ++c)
                    if (c < COPIES_PER_WAVE && more) copy_nth(tc, c);
            });
            st_v = st_v + 1 < NSTAGE ? st_v + 1 : 0;
        }
    }

    // ---- epilogue ----------------------------------------------------------------------------------
    if (scorer) {
        const float l_lane = l_run + xor32(l_run);
        const float lr_lane = lr_run + xor32(lr_run);
        if (lh == 0) {
            s_lpart[wr * 32 + ln] = l_lane;
            s_lpart[M + wr * 32 + ln] = lr_lane;
        }
    }
    lds_barrier();

    if (!DECODE && !PRECISE) {
        // A result of magnitude 2 or more leaves the error budget little beyond its own rounding to
        // bf16 (half an ulp is 2^-7 there), and it can only come from a row whose weight sits on a few
        // keys, where the rounding of P to bf16 shows most. A tile with such a row is not written: it
        // is computed again with two-term P (the caller runs the PRECISE pass when this one says so).
        bool big = false;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const float rsum = s_lpart[M + rb * 32 + ln];
            float mx = 0.f;
#pragma unroll
            for (int db = 0; db < C::DVB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, __builtin_fabsf(o[db][rb][e]));
            big = big || (rsum > 0.f && mx >= kRedoMagnitude * rsum && r0 + rb * 32 + ln < R);
        }
        if (__any(big) && lane == 0) *s_redo = 1;
        lds_barrier();
        if (*(volatile int *)s_redo) return true;
    }

    if (!DECODE) {
        // lse = ln(sum_j exp(scale q.k_j)) = (m_ref + log2 l) * ln 2
        if (scorer && lh == 0 && my_row < R) {
            const int hh = (int)(my_row - (int64_t)r_row * G);
            p.lse[((int64_t)b * p.Hq + (int64_t)g * G + hh) * Sq + r_row] =
                (m_ref + __builtin_amdgcn_logf(s_lpart[wr * 32 + ln])) * 0.69314718055994530942f;
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int64_t row = r0 + rb * 32 + ln;
            const float rsum = s_lpart[M + rb * 32 + ln];
            const float inv = rsum > 0.f ? 1.0f / rsum : 0.f;  // a row without a live key gives 0
            if (row < R) {
                const int64_t i = row / G;
                const int hh = (int)(row - i * G);
                const int64_t o_idx = ((((int64_t)b * Sq + i) * p.Hq + (int64_t)g * G + hh) * DV) + vw * C::DVW + 4 * lh;
                if constexpr (OUTF32) {
                    // unrounded output (the calibration blend rounds once, after mixing two of these)
                    float *op = p.out_f32 + o_idx;
#pragma unroll
                    for (int db = 0; db < C::DVB; ++db)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            float4 w;
                            w.x = o[db][rb][4 * qd + 0] * inv;
                            w.y = o[db][rb][4 * qd + 1] * inv;
                            w.z = o[db][rb][4 * qd + 2] * inv;
                            w.w = o[db][rb][4 * qd + 3] * inv;
                            *(float4 *)(op + db * 32 + qd * 8) = w;
                        }
                } else {
                    uint16_t *op = p.out + o_idx;
#pragma unroll
                    for (int db = 0; db < C::DVB; ++db)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            u32x2 w;
                            w[0] = pack_bf16(o[db][rb][4 * qd + 0] * inv, o[db][rb][4 * qd + 1] * inv);
                            w[1] = pack_bf16(o[db][rb][4 * qd + 2] * inv, o[db][rb][4 * qd + 3] * inv);
                            *(u32x2 *)(op + db * 32 + qd * 8) = w;
                        }
                }
            }
        }
    } else {
        // partial result of this key split: unnormalised O (relative to m_ref), m_ref, l, rounded l
        if (scorer && lh == 0 && my_row < R) {
            const int64_t h = (int64_t)b * p.Hq + (int64_t)g * G + my_row;
            p.part_ml[(h * p.n_splits + split) * 4 + 0] = m_ref;
            p.part_ml[(h * p.n_splits + split) * 4 + 1] = s_lpart[wr * 32 + ln];
            p.part_ml[(h * p.n_splits + split) * 4 + 2] = s_lpart[M + wr * 32 + ln];
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int64_t row = r0 + rb * 32 + ln;
            if (!scorer && row < R) {
                const int64_t h = (int64_t)b * p.Hq + (int64_t)g * G + row;
                float *op = p.part_o + (h * p.n_splits + split) * DV + vw * C::DVW + 4 * lh;
#pragma unroll
                for (int db = 0; db < C::DVB; ++db)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        float4 w;
                        w.x = o[db][rb][4 * qd + 0];
                        w.y = o[db][rb][4 * qd + 1];
                        w.z = o[db][rb][4 * qd + 2];
                        w.w = o[db][rb][4 * qd + 3];
                        *(float4 *)(op + db * 32 + qd * 8) = w;
                    }
            }
        }
    }
    return false;
}

// Prefill / extend: every tile is computed with P rounded to bf16 once; a tile that cannot afford
// that (few live keys per row, or a result large enough that its own rounding fills the error
// budget) is computed with two-term P instead. Decode: one pass of the split kernel.
template <int DQK, int DV, int RB, bool ALIAS, bool DECODE, bool OUTF32 = false, bool EXT = false>
__global__ __launch_bounds__(256) void ssa_fwd_kernel(const FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    if constexpr (DECODE) {
        ssa_fwd_tile<DQK, DV, RB, ALIAS, true, false, false, false>(p, smem);
    } else {
        if (ssa_fwd_tile<DQK, DV, RB, ALIAS, false, false, OUTF32, EXT>(p, smem))
            ssa_fwd_tile<DQK, DV, RB, ALIAS, false, true, OUTF32, EXT>(p, smem);
    }
}

// One decode query computed from the cache rows themselves: scores, softmax and weighted sum in fp32
// (no rounding of the weights). All threads of the workgroup (one per four output columns) call it
// together. The live keys are walked twice, in chunks of kDirectKeys: once for the maximum of the
// scores, once for the weights and the weighted sum (a query whose keys fit one chunk keeps its
// scores between the two). n_live >= 1.
template <int DQK, int DV>
static __device__ void decode_row_direct(const FwdParams &p, int64_t h, int b, int g, int64_t se, int64_t wb, int64_t n_live)
{
    constexpr int NT = DV / 4;
    __shared__ float s_w[kDirectKeys];
    __shared__ __attribute__((aligned(16))) float s_q[DQK];
    __shared__ float s_m[NT];
    const int tid = threadIdx.x, c = tid * 4;
    const int64_t k_step = (int64_t)p.Hkv * DQK;
    const bool alias = (p.v == p.k);
    const int64_t v_step = (int64_t)p.Hkv * (alias ? DQK : DV);
    const bool paged = p.block_table != nullptr;
    const int64_t seq_row0 = paged ? 0 : (int64_t)b * p.S;
    const uint16_t *kb = p.k + (seq_row0 * p.Hkv + g) * DQK;
    const uint16_t *vb = p.v + (seq_row0 * p.Hkv + g) * (alias ? DQK : DV);
    // cache row of the t-th live key (through the block table of a paged cache)
    auto key_of = [&](int64_t t) {
        const int64_t j = t < se ? t : wb + (t - se);
        if (!paged) return j;
        int pid = p.block_table[(int64_t)b * p.max_pages + (j >> p.page_shift)];
        pid = pid < 0 ? 0 : (pid < p.num_pages ? pid : p.num_pages - 1);
        return ((int64_t)pid << p.page_shift) + (j & ((1 << p.page_shift) - 1));
    };
    auto lo16 = [](uint32_t w) { return __builtin_bit_cast(float, w << 16); };
    auto hi16 = [](uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); };
    const uint16_t *q = p.q + h * DQK;
    for (int e = tid; e < DQK; e += NT) s_q[e] = __builtin_bit_cast(float, (uint32_t)q[e] << 16);
    __syncthreads();
    // scale * log2(e) * q . k of the t-th live key
    auto score = [&](int64_t t) {
        const u32x4 *kr = (const u32x4 *)(kb + key_of(t) * k_step);
        float dot = 0.f;
#pragma unroll 2
        for (int c8 = 0; c8 < DQK / 8; ++c8) {
            const u32x4 w = kr[c8];
            const float4 qa = *(const float4 *)(s_q + 8 * c8), qb = *(const float4 *)(s_q + 8 * c8 + 4);
            dot = __builtin_fmaf(qa.x, lo16(w[0]), dot);
            dot = __builtin_fmaf(qa.y, hi16(w[0]), dot);
            dot = __builtin_fmaf(qa.z, lo16(w[1]), dot);
            dot = __builtin_fmaf(qa.w, hi16(w[1]), dot);
            dot = __builtin_fmaf(qb.x, lo16(w[2]), dot);
            dot = __builtin_fmaf(qb.y, hi16(w[2]), dot);
            dot = __builtin_fmaf(qb.z, lo16(w[3]), dot);
            dot = __builtin_fmaf(qb.w, hi16(w[3]), dot);
        }
        return dot * p.scale_log2;
    };
    const bool one_chunk = n_live <= kDirectKeys;
    float m = LOZA_NEG_INF;
    for (int64_t t = tid; t < n_live; t += NT) {
        const float sc = score(t);
        if (one_chunk) s_w[t] = sc;
        m = fmaxf(m, sc);
    }
    s_m[tid] = m;
    __syncthreads();
    for (int t = 0; t < NT; ++t) m = fmaxf(m, s_m[t]);
    float l = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t c0 = 0; c0 < n_live; c0 += kDirectKeys) {
        const int cnt = (int)(n_live - c0 < kDirectKeys ? n_live - c0 : kDirectKeys);
        for (int t = tid; t < cnt; t += NT) s_w[t] = __builtin_amdgcn_exp2f((one_chunk ? s_w[t] : score(c0 + t)) - m);
        __syncthreads();
        for (int t = 0; t < cnt; ++t) {
            const float w = s_w[t];
            const u32x2 vr = *(const u32x2 *)(vb + key_of(c0 + t) * v_step + c);
            l += w;
            acc.x = __builtin_fmaf(w, lo16(vr[0]), acc.x);
            acc.y = __builtin_fmaf(w, hi16(vr[0]), acc.y);
            acc.z = __builtin_fmaf(w, lo16(vr[1]), acc.z);
            acc.w = __builtin_fmaf(w, hi16(vr[1]), acc.w);
        }
        __syncthreads();
    }
    const float inv = 1.0f / l;
    u32x2 w2;
    w2[0] = pack_bf16(acc.x * inv, acc.y * inv);
    w2[1] = pack_bf16(acc.z * inv, acc.w * inv);
    *(u32x2 *)(p.out + h * DV + c) = w2;
    if (tid == 0) p.lse[h] = (m + __builtin_amdgcn_logf(l)) * 0.69314718055994530942f;
}

// Merge of the key splits of one decode query (log-sum-exp rule, fixed split order). Each split s
// left O_s (unnormalised, relative to its reference m_s), the sum l_s of its exponentials and the
// sum r_s of the same values as rounded to bf16 (what O_s was accumulated from):
//   m* = max_s m_s ;  w_s = 2^(m_s - m*) ;  out = sum_s w_s O_s / sum_s w_s r_s ;
//   lse = (m* + log2 sum_s w_s l_s) ln 2.
// One workgroup per (sequence, query head), one thread per four output columns. Two kinds of query
// are computed here from the cache rows instead (decode_row_direct): one with fewer than kDirectKeys
// live keys, which never went through the split kernel, and one whose merged result reaches
// kRedoMagnitude in some column (the weights of the split kernel are rounded to bf16, which a result
// that large cannot afford).
template <int DQK, int DV>
__global__ __launch_bounds__(DV / 4) void ssa_decode_merge_kernel(const FwdParams p)
{
    const int64_t h = blockIdx.x;  // flat (b, query head)
    const int c = threadIdx.x * 4;
    const int n_splits = p.n_splits;
    uint16_t *out = p.out + h * DV + c;

    const int b = (int)(h / p.Hq), hq = (int)(h - (int64_t)b * p.Hq), g = hq / p.G;
    const int64_t L = (int64_t)p.seqlens[b] < p.S ? (int64_t)p.seqlens[b] : p.S;
    const int64_t se = p.n_sink < L ? p.n_sink : L;
    int64_t wb = L > 0 ? window_begin_of((int)(L - 1), p.window, p.block) : 0;
    if (wb < se) wb = se;
    const int64_t n_live = se + (L - wb);
    if (n_live <= 0) {  // empty cache
        u32x2 z; z[0] = 0; z[1] = 0;
        *(u32x2 *)out = z;
        if (threadIdx.x == 0) p.lse[h] = LOZA_NEG_INF;
        return;
    }
    if (n_live < kDirectKeys) {
        decode_row_direct<DQK, DV>(p, h, b, g, se, wb, n_live);
        return;
    }

    // ---- merge of the key splits -------------------------------------------------------------------
    const float *ml = p.part_ml + h * n_splits * 4;
    float m_star = LOZA_NEG_INF;
    for (int s = 0; s < n_splits; ++s) m_star = fmaxf(m_star, ml[4 * s]);
    float den = 0.f, den_r = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < n_splits; ++s) {
        const float w = __builtin_amdgcn_exp2f(ml[4 * s] - m_star);
        den += w * ml[4 * s + 1];
        den_r += w * ml[4 * s + 2];
        const float4 v = *(const float4 *)(p.part_o + (h * n_splits + s) * DV + c);
        acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
    }
    const float inv = 1.0f / den_r;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    const bool big = fmaxf(fmaxf(__builtin_fabsf(acc.x), __builtin_fabsf(acc.y)), fmaxf(__builtin_fabsf(acc.z), __builtin_fabsf(acc.w))) >= kRedoMagnitude;
    if (__syncthreads_or(big)) {
        decode_row_direct<DQK, DV>(p, h, b, g, se, wb, n_live);
        return;
    }
    u32x2 w2;
    w2[0] = pack_bf16(acc.x, acc.y);
    w2[1] = pack_bf16(acc.z, acc.w);
    *(u32x2 *)out = w2;
    if (threadIdx.x == 0) p.lse[h] = (m_star + __builtin_amdgcn_logf(den)) * 0.69314718055994530942f;
}

// ---------------------------------------------------------------------------------------------------

// A pattern that leaves rows beyond the first kPrecisePositions positions with fewer live keys than
// that takes the two-term variant throughout. The smallest live set of such a row is at position
// kPrecisePositions - 1 or at the first query of a block whose window has reached full length.
static bool pattern_needs_precise(const FwdParams &p)
{
    auto live_at = [&](int64_t i) {
        const int64_t se = p.n_sink < i + 1 ? p.n_sink : i + 1;
        const int64_t qb = i / p.block;
        int64_t wb = p.window > qb ? 0 : (qb - p.window + 1) * p.block;
        if (wb < se) wb = se;
        return se + (i + 1 - wb);
    };
    if (p.S < kPrecisePositions) return false;
    int64_t qb0 = (kPrecisePositions - 1 + p.block - 1) / p.block;
    if (qb0 < p.window - 1) qb0 = p.window - 1;
    const int64_t i0 = qb0 * p.block;
    return live_at(kPrecisePositions - 1) < kPrecisePositions || (i0 < p.S && live_at(i0) < kPrecisePositions);
}

// The tile kernels use more dynamic LDS than the default limit: raised once per kernel and device.
template <auto KERN>
static hipError_t allow_lds(int bytes)
{
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute((const void *)KERN, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done[dev] = true;
    return e;
}

template <int DQK, int DV, bool ALIAS, bool OUTF32, bool EXT>
static hipError_t launch_prefill_kernel(FwdParams p, hipStream_t stream)
{
    using C = TileCfg<DQK, DV, 4, ALIAS, false>;
    constexpr auto kern = ssa_fwd_kernel<DQK, DV, 4, ALIAS, false, OUTF32, EXT>;
    hipError_t e = allow_lds<kern>(C::LDS_BYTES);
    if (e != hipSuccess) return e;
    p.rt_begin = 0;
    p.all_precise = pattern_needs_precise(p) ? 1 : 0;
    // The speculative softmax scores a tile twice when the reference moves: the reference is exact
    // over the first tile only, afterwards lazy (with an exact reference over the first 8 tiles most
    // of them would move it).
    if (C::SPEC_SOFTMAX) p.exact_tiles = 1;
    const int64_t blocks = (int64_t)p.row_tiles * p.Hkv * p.B;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <int DQK, int DV, bool ALIAS>
static hipError_t launch_prefill_t(const FwdParams &p, hipStream_t stream)
{
    if (p.out_f32 != nullptr) return launch_prefill_kernel<DQK, DV, ALIAS, true, false>(p, stream);
    return launch_prefill_kernel<DQK, DV, ALIAS, false, false>(p, stream);
}

// Extend prefill: the same kernel in the form that takes its positions from the sequence lengths
template <int DQK, int DV, bool ALIAS>
static hipError_t launch_extend_t(const FwdParams &p, hipStream_t stream)
{
    return launch_prefill_kernel<DQK, DV, ALIAS, false, true>(p, stream);
}

template <int DQK, int DV, bool ALIAS>
static hipError_t launch_decode_t(const FwdParams &p, hipStream_t stream)
{
    using C = TileCfg<DQK, DV, 2, ALIAS, true>;
    constexpr auto kern = ssa_fwd_kernel<DQK, DV, 2, ALIAS, true>;
    hipError_t e = allow_lds<kern>(C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int64_t blocks = (int64_t)p.n_splits * p.row_tiles * p.Hkv * p.B;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((ssa_decode_merge_kernel<DQK, DV>), dim3((unsigned)((int64_t)p.B * p.Hq)), dim3(DV / 4), 0, stream, p);
    return hipGetLastError();
}

// Calibration blend (paper: Architecture section, Eq. 3): out = alpha * o_full + (1 - alpha) * o_sparse,
// element-wise on the unrounded fp32 outputs of two prefill launches, rounded to bf16 once. The two
// inputs can be written out rounded as well (either pointer may be null). n is a multiple of 4.
__global__ __launch_bounds__(256) void ssa_blend_kernel(const float *__restrict__ o_full, const float *__restrict__ o_sparse,
                                                        float alpha, uint16_t *__restrict__ out,
                                                        uint16_t *__restrict__ out_full, uint16_t *__restrict__ out_sparse,
                                                        int64_t n4)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const float4 a = ((const float4 *)o_full)[i], s = ((const float4 *)o_sparse)[i];
        const float beta = 1.0f - alpha;
        u32x2 w;
        w[0] = pack_bf16(__builtin_fmaf(alpha, a.x, beta * s.x), __builtin_fmaf(alpha, a.y, beta * s.y));
        w[1] = pack_bf16(__builtin_fmaf(alpha, a.z, beta * s.z), __builtin_fmaf(alpha, a.w, beta * s.w));
        ((u32x2 *)out)[i] = w;
        if (out_full) { w[0] = pack_bf16(a.x, a.y); w[1] = pack_bf16(a.z, a.w); ((u32x2 *)out_full)[i] = w; }
        if (out_sparse) { w[0] = pack_bf16(s.x, s.y); w[1] = pack_bf16(s.z, s.w); ((u32x2 *)out_sparse)[i] = w; }
    }
}

hipError_t launch_blend_bf16(const float *o_full, const float *o_sparse, float alpha, uint16_t *out,
                             uint16_t *out_full, uint16_t *out_sparse, int64_t n, hipStream_t stream)
{
    const int64_t n4 = n / 4;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;  // grid-stride beyond that
    hipLaunchKernelGGL(ssa_blend_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, o_full, o_sparse, alpha, out,
                       out_full, out_sparse, n4);
    return hipGetLastError();
}

// Gradient of the calibration blend with respect to alpha (paper: Architecture section, Eq. 3):
// d/d(alpha) [alpha O + (1 - alpha) O'] = O - O', so d(alpha) = sum over every element of
// dout * (O - O'), from the bf16 tensors the blend wrote. Two launches and a fixed order of
// addition (deterministic): per-workgroup partial sums in fp64, then one workgroup adds those.
constexpr int kAlphaGradBlocks = 4096;

static __device__ __forceinline__ double block_sum_256(double x, double *sm)
{
    sm[threadIdx.x] = x;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sm[threadIdx.x] += sm[threadIdx.x + s];
        __syncthreads();
    }
    return sm[0];
}

__global__ __launch_bounds__(256) void ssa_alpha_grad_partial_kernel(const uint16_t *__restrict__ dout, const uint16_t *__restrict__ o_full,
                                                                     const uint16_t *__restrict__ o_sparse, double *__restrict__ partial,
                                                                     int64_t n8)
{
    __shared__ double sm[256];
    auto widen = [](uint32_t bits) { return (double)__builtin_bit_cast(float, bits); };
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const u32x4 d = ((const u32x4 *)dout)[i], a = ((const u32x4 *)o_full)[i], s = ((const u32x4 *)o_sparse)[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += widen(d[e] << 16) * (widen(a[e] << 16) - widen(s[e] << 16));
            acc += widen(d[e] & 0xffff0000u) * (widen(a[e] & 0xffff0000u) - widen(s[e] & 0xffff0000u));
        }
    }
    const double total = block_sum_256(acc, sm);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void ssa_alpha_grad_final_kernel(const double *__restrict__ partial, int n_partial, float *__restrict__ dalpha)
{
    __shared__ double sm[256];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n_partial; i += 256) acc += partial[i];
    const double total = block_sum_256(acc, sm);
    if (threadIdx.x == 0) *dalpha = (float)total;
}

int alpha_grad_blocks(int64_t n)
{
    const int64_t n8 = n / 8, b = (n8 + 255) / 256;
    return (int)(b < kAlphaGradBlocks ? (b < 1 ? 1 : b) : kAlphaGradBlocks);
}

hipError_t launch_alpha_grad_bf16(const uint16_t *dout, const uint16_t *o_full, const uint16_t *o_sparse, float *dalpha, int64_t n,
                                  double *partial, hipStream_t stream)
{
    const int blocks = alpha_grad_blocks(n);
    hipLaunchKernelGGL(ssa_alpha_grad_partial_kernel, dim3(blocks), dim3(256), 0, stream, dout, o_full, o_sparse, partial, n / 8);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ssa_alpha_grad_final_kernel, dim3(1), dim3(256), 0, stream, (const double *)partial, blocks, dalpha);
    return hipGetLastError();
}

bool bf16_shape_supported(int d_qk, int d_v, bool alias)
{
    if (d_qk == 576 && d_v == 512) return alias;
    if (d_qk == 128 && d_v == 128) return true;
    return false;
}

int prefill_rows_per_tile() { return 128; }
int decode_rows_per_tile() { return 64; }

hipError_t launch_prefill_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream)
{
    if (d_qk == 576 && d_v == 512 && alias) return launch_prefill_t<576, 512, true>(p, stream);
    if (d_qk == 128 && d_v == 128) return alias ? launch_prefill_t<128, 128, true>(p, stream)
                                                : launch_prefill_t<128, 128, false>(p, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_extend_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream)
{
    if (d_qk == 576 && d_v == 512 && alias) return launch_extend_t<576, 512, true>(p, stream);
    if (d_qk == 128 && d_v == 128) return alias ? launch_extend_t<128, 128, true>(p, stream)
                                                : launch_extend_t<128, 128, false>(p, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_decode_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream)
{
    if (d_qk == 576 && d_v == 512 && alias) return launch_decode_t<576, 512, true>(p, stream);
    if (d_qk == 128 && d_v == 128) return alias ? launch_decode_t<128, 128, true>(p, stream)
                                                : launch_decode_t<128, 128, false>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace loza

