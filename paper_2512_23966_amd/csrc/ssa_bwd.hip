// Backward of bf16 streaming sparse attention for gfx950 (MI355X): dQ, dK, dV over live tiles only.
//
// What is computed (the derivative of the paper's Eq. 4 that its sparse mid-training needs;
// Architecture section, Training paragraph): with O = softmax(scale Q K*^T) V* over the live key set
// of every query, lse the log of the softmax denominator and dO the gradient arriving at O,
//   p_ij  = exp(scale q_i.k_j - lse_i)  (live j),   D_i = dO_i . O_i
//   dV_j  = sum_i p_ij dO_i             dP_ij = dO_i . v_j        dS_ij = p_ij (dP_ij - D_i)
//   dQ_i  = scale sum_j dS_ij k_j       dK_j  = scale sum_i dS_ij q_i
// where the sums over i run over every query row (all heads of the key's group) that sees key j.
// When the values are a prefix of the key rows (absorbed MLA: one latent serves both), the gradient
// of that one tensor is dK with dV added to its first d_v columns, and that sum is what is written.
//
// Three kernels:
//   * ssa_bwd_rowstat_kernel: per query row, (lse log2(e), D) in the row order the main kernel
//     walks through (position-major, heads of a group together).
//   * ssa_bwd_kernel<.., KEYS = false>: one workgroup keeps 64 query rows (Q and dO as matrix-core
//     operands in registers) and streams the live key tiles of 32 keys past them: dQ.
//   * ssa_bwd_kernel<.., KEYS = true>: one workgroup keeps 64 keys (K and V in registers) and
//     streams the tiles of 32 query rows that see them: dK and dV. A key tile that holds sink keys
//     is seen by every later query; its rows are cut into chunks that run as workgroups of their own
//     and leave fp32 partial sums, which ssa_bwd_reduce_kernel adds in chunk order.
// Both forms of the main kernel are the same program with the roles of rows and keys exchanged:
//   stationary side X (two blocks of 32), streamed side Y (tiles of 32), and per tile
//     phase 1:  S[y][x] = Y1 X1^T (contraction d_qk)   and   T[y][x] = Y2 X2^T (contraction d_v)
//               on different wavefronts (S: waves 0, 1; T: waves 2, 3; one block of X each); the
//               two waves of a block swap halves of their results through LDS and each forms p
//               and dS for its half, left as bf16 in LDS ([x][y], y contiguous);
//     phase 2:  Acc^T[d][x] += Y^T[d][y] dS[y][x]  (and += Y2^T p for dV), all four waves, each
//               owning a few blocks of 32 columns for both blocks of X; the streamed tile is read
//               transposed from LDS (ds_read_b64_tr_b16) as the forward's value phase does, and
//               every fragment read feeds two matrix instructions.
// The streamed tiles travel global -> LDS with global_load_lds_dwordx4 into a ring of two stages,
// the copy instructions of the next tile issued between the matrix instructions of phase 1 (a copy
// requested later than that is still on its way when the next iteration needs it).
// After the setup the two roles run separate instantiations of the tile loop.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "score_asm.h"
#include "ssa_device.h"
#include "ssa_kernels.h"

namespace loza {

namespace {

// One global -> LDS copy instruction: 64 lanes x 16 bytes from base + off (per lane) to the 1 KB of
// LDS at lds_addr (wave-uniform, through M0). The compiler's wait counters do not see it: the tile
// loop waits for all of them (vmcnt(0)) before the barrier that publishes a tile.
__device__ __forceinline__ void copy_1k(const char *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n s_nop 0\n global_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_addr) : "memory", "m0");
}

// Matrix-core A operand [32 columns of block db][16 items of key step ks] of a tile stored
// [item][column] (padded rows of `row` bytes): two transposing 64-bit reads.
__device__ __forceinline__ bf16x8 read_transposed(const char *tile, int row, int db, int ks, int lane)
{
    const int lh = lane >> 5, s16 = lane & 15, g16 = (lane >> 4) & 1;
    const char *a = tile + (ks * 16 + lh * 8 + (s16 >> 2)) * row + (db * 32 + g16 * 16 + (s16 & 3) * 4) * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a + 4 * row));
    s16x8 a8;
    a8[0] = lo[0]; a8[1] = lo[1]; a8[2] = lo[2]; a8[3] = lo[3];
    a8[4] = hi[0]; a8[5] = hi[1]; a8[6] = hi[2]; a8[7] = hi[3];
    return __builtin_bit_cast(bf16x8, a8);
}

}  // namespace

// (lse log2(e), dO . O) of every query row, stored [B, Hkv, Rpad] with row index i * G + head-in-group.
template <int DV>
__global__ __launch_bounds__(256) void ssa_bwd_rowstat_kernel(const BwdParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // flat (b, i, h)
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq;
    if (row >= n_rows) return;
    const uint16_t *o = p.out + row * DV, *d = p.dout + row * DV;
    float acc = 0.f;
    for (int c = lane * 8; c < DV; c += 512) {
        const u32x4 a = *(const u32x4 *)(o + c), b = *(const u32x4 *)(d + c);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = __builtin_fmaf(__builtin_bit_cast(float, a[e] << 16), __builtin_bit_cast(float, b[e] << 16), acc);
            acc = __builtin_fmaf(__builtin_bit_cast(float, a[e] & 0xffff0000u), __builtin_bit_cast(float, b[e] & 0xffff0000u), acc);
        }
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) acc += __shfl_xor(acc, s, 64);
    if (lane == 0) {
        const int h = (int)(row % p.Hq);
        const int64_t bi = row / p.Hq, i = bi % p.S, b = bi / p.S;
        const int g = h / p.G, hh = h - g * p.G;
        float2 st;
        st.x = p.lse[(b * p.Hq + h) * p.S + i] * 1.44269504088896340736f;
        st.y = acc;
        p.rowstat[(b * p.Hkv + g) * p.r_pad + i * p.G + hh] = st;
    }
}

template <int DQK, int DV, bool ALIAS, bool KEYS>
struct BwdCfg {
    static constexpr int ROW1 = DQK * 2 + 16, ROW2 = DV * 2 + 16;   // padded LDS rows of the streamed tiles
    static constexpr int CPR1 = ROW1 / 16, CPR2 = ROW2 / 16;
    static constexpr bool HAS_Y2 = KEYS || !ALIAS;    // a second streamed tile (dO rows, or separate values)
    static constexpr int N1 = (32 * CPR1 + 63) / 64;  // 1 KB copy instructions per tile
    static constexpr int N2 = HAS_Y2 ? (32 * CPR2 + 63) / 64 : 0;
    static constexpr int NSTAT = KEYS ? 1 : 0;        // + the row statistics of the tile
    static constexpr int NI = N1 + N2 + NSTAT;
    // Who copies what: instruction c * 4 + w of a sub-tile belongs to wave w for c < A1 (A2); what is
    // left over (at most one instruction per wave: the tails of the two sub-tiles and the statistics)
    // is dealt one to a wave as its last, "extra" instruction. Every wave thus issues the same
    // sequence: A1 into the first sub-tile, A2 into the second, and possibly one more.
    static constexpr int A1 = N1 / 4, A2 = N2 / 4, R1 = N1 % 4, R2 = N2 % 4;
    static constexpr int NEXTRA = R1 + R2 + NSTAT;
    static_assert(NEXTRA <= 4, "one extra copy instruction per wave at most");
    static constexpr int PER_WAVE = A1 + A2 + 1;
    // Wide rows, key-stationary kernel: 18 copy instructions per wave between the 36 matrix instructions
    // of phase 1 are more than the compute unit's memory pipeline takes at that pace (the waves queue
    // on it); only A2_WOVEN of the second sub-tile's are woven into phase 1, the others go out in pairs
    // during the elementwise step (measured: in threes slightly worse, in fours much worse).
    static constexpr int A2_WOVEN = (KEYS && DQK == 576 && DV == 512) ? 2 : A2;
    static constexpr int STAGE = NI * 1024;
    static constexpr int OFF_Y2 = N1 * 1024, OFF_STAT = (N1 + N2) * 1024;
    static constexpr int PROW = 32 * 2 + 16;          // LDS bytes per row of the dS / p buffers
    static constexpr int XREGION = 2 * 32 * PROW;     // per block of X: dS rows, then p rows
    static constexpr int XCH = 64 * 16 * 4;           // per block of X: the T block handed over, fp32
    static constexpr int OFF_BUF = 2 * STAGE;
    static constexpr int OFF_XCH = OFF_BUF + 2 * XREGION;
    static constexpr int LDS_BYTES = OFF_XCH + 2 * XCH;
    static_assert(LDS_BYTES <= 160 * 1024, "does not fit the 160 KB LDS");
    // accumulator blocks (32 columns x 32 items of X) per wave
    static constexpr bool SPLIT_KV = KEYS && !ALIAS;  // half the waves take dK, the other half dV
    static_assert(!SPLIT_KV || DQK == DV, "separate values: equal widths only");
    // Phase 2: every wave accumulates a few column blocks (32 columns) for BOTH blocks of X, so that a
    // transposed fragment of the streamed tile, once fetched from LDS, feeds two matrix instructions
    // (fetched once per block of X, LDS bandwidth bounds the kernel). ND0 / ND1: column blocks of a
    // wave of role 0 / role 1; role 0 (longer phase 1, four more operand fragments) takes the smaller share.
    static constexpr int NBLK = DQK / 32;
    static constexpr int ND0 = SPLIT_KV ? NBLK / 2 : NBLK / 4;
    static constexpr int ND1 = SPLIT_KV ? (DV / 32) / 2 : (NBLK - 2 * ND0) / 2;
    static_assert(SPLIT_KV || 2 * ND0 + 2 * ND1 == NBLK, "column blocks must split over the four waves");
    // of a role-1 wave's blocks, how many also take the second product (dV, columns below d_v)
    static constexpr int NDBL1 = (KEYS && !SPLIT_KV) ? (DV / 32 - 2 * ND0) / 2 : 0;
    static_assert(NDBL1 >= 0 && NDBL1 <= ND1, "split of the d_v columns");
    static_assert(DQK % 64 == 0 && DV % 32 == 0 && DV <= DQK, "head widths");
};

template <int DQK, int DV, bool ALIAS, bool KEYS>
__global__ __launch_bounds__(256) void ssa_bwd_kernel(const BwdParams p)
{
    using C = BwdCfg<DQK, DV, ALIAS, KEYS>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const uint32_t smem_lds = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)smem);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, ln = lane & 31, lh = lane >> 5;
    const int xb = wave & 1, role = wave >> 1;  // role 0: S = Y1 X1^T; role 1: T = Y2 X2^T; the elementwise step is shared
    const int G = p.G;
    const int64_t S = p.S, R = S * G;
    const int n_sink = p.n_sink, window = p.window, block = p.block;
    // Row index -> position, once or twice per tile: a shift when the group size is a power of two
    // (an integer division by a run-time value is dozens of dependent instructions on a wave that
    // has nothing else to issue meanwhile).
    const int g_log2 = (G & (G - 1)) == 0 ? __builtin_ctz((unsigned)G) : -1;
    auto div_g = [&](int r) { return g_log2 >= 0 ? r >> g_log2 : r / G; };

    // ---- which work item ----------------------------------------------------------------------------
    const int n_kt = (int)((S + 63) / 64);  // key tiles of 64 keys
    int b, g, xt, chunk = 0;
    bool partial = false;  // KEYS: leave an fp32 partial sum for the reduce kernel
    if (!KEYS) {
        const int x_tiles = (int)((R + 63) / 64);
        int id = blockIdx.x;
        xt = x_tiles - 1 - id % x_tiles;  // latest (heaviest) rows first
        id /= x_tiles;
        g = id % p.Hkv;
        b = id / p.Hkv;
    } else {
        const int items = p.n_sink_kt * p.max_chunks + (n_kt - p.n_sink_kt);
        // Workgroups go to the eight XCDs round-robin and every XCD has an L2 of its own. Handing every
        // XCD one contiguous eighth of the items makes the workgroups that share an L2 neighbouring key
        // tiles, whose row ranges overlap almost completely (see the rotation below).
        int id = blockIdx.x;
        {
            const int total = gridDim.x, eighth = total / 8;
            if (id < eighth * 8) id = (id % 8) * eighth + id / 8;
        }
        const int it = id % items;
        id /= items;
        g = id % p.Hkv;
        b = id / p.Hkv;
        if (it < p.n_sink_kt * p.max_chunks) {
            xt = it / p.max_chunks;
            chunk = it % p.max_chunks;
            partial = p.max_chunks > 1;
        } else {
            xt = p.n_sink_kt + (it - p.n_sink_kt * p.max_chunks);
        }
    }

    // ---- streamed tiles of this item -------------------------------------------------------------
    // !KEYS: the live key tiles of rows [xt*64, xt*64+64): sink tiles [0, nA), then window tiles.
    // KEYS: the row tiles [yt_begin, yt_begin + nt) that can see keys [xt*64, xt*64+64).
    int nt, nA = 0, wt0 = 0, yt_begin = 0, yt_start = 0;
    int i_min = 0, i_max = 0, w_lo_max = 0;
    if (!KEYS) {
        const int64_t r_last = (int64_t)xt * 64 + 63 < R ? (int64_t)xt * 64 + 63 : R - 1;
        i_min = (int)(((int64_t)xt * 64) / G);
        i_max = (int)(r_last / G);
        const int sink_end = n_sink < i_max + 1 ? n_sink : i_max + 1;
        const int win_begin = window_begin_of(i_min, window, block);
        w_lo_max = window_begin_of(i_max, window, block);
        nA = (sink_end + 31) / 32;
        wt0 = win_begin / 32;
        const int wt1 = i_max / 32;
        int nB;
        if (wt0 <= nA) { nA = wt1 + 1; nB = 0; } else { nB = wt1 - wt0 + 1; }
        nt = nA + nB;
    } else {
        int yt_lo, yt_hi;
        bwd_key_tile_rows(p, xt, yt_lo, yt_hi);
        yt_begin = yt_lo;
        int yt_end = yt_hi + 1;
        if (xt < p.n_sink_kt) {
            yt_begin = yt_lo + chunk * p.chunk_tiles;
            if (yt_begin + p.chunk_tiles < yt_end) yt_end = yt_begin + p.chunk_tiles;
        }
        nt = yt_end - yt_begin;
        if (nt <= 0) return;  // a chunk beyond the rows of this key tile (the reduce kernel knows)
        // Neighbouring key tiles see almost the same rows, each range shifted by 64 positions. Left to
        // start at its own first row tile, every workgroup would stream its q and dout rows at a
        // different place at any moment, and all of it would come from HBM (at the 128K shape: 2.4 TB
        // per launch). Instead the 32 key tiles of a group (the workgroups that run together on one
        // XCD) all start at the first row tile of the group's last member and wrap around inside their
        // own range: they then ask for the same row tile at about the same time, and one fetch into
        // the shared L2 serves all of them.
        yt_start = yt_begin;
        if (xt >= p.n_sink_kt) {
            const int last = p.n_sink_kt + ((xt - p.n_sink_kt) / 32) * 32 + 31;
            int a_lo, a_hi;
            bwd_key_tile_rows(p, last < n_kt - 1 ? last : n_kt - 1, a_lo, a_hi);
            if (a_lo >= yt_begin && a_lo < yt_end) yt_start = a_lo;
        }
    }
    const int yt_wrap = yt_begin + nt;
    auto y_tile = [&](int t) {
        if (!KEYS) return t < nA ? t : wt0 + (t - nA);
        const int yt = yt_start + t;
        return yt < yt_wrap ? yt : yt - nt;
    };

    // KEYS: the row tiles that need no mask are a contiguous run. A tile starting at row y0 (rows
    // y0 .. y0 + 31, positions i_lo = y0 / G .. i_hi = (y0 + 31) / G) is interior when all its rows
    // exist, all 64 keys exist, the last key is not after the first position (j_max <= i_lo), and
    // either all keys are sinks or the first key is inside the window of the last position
    // (j_min >= window_begin(i_hi), which does not decrease with the position).
    int y_int_lo = 1, y_int_hi = 0;  // (empty)
    if (KEYS) {
        const int64_t j_min = (int64_t)xt * 64, j_max = j_min + 63;
        if (j_max < S) {
            // j_max <= y0 / G  <=>  y0 >= j_max * G
            const int64_t lo = j_max * G;
            // rows exist: y0 + 31 < R
            int64_t hi = R - 32;
            if (j_max >= n_sink) {
                // window_begin(i) <= j_min  <=>  i / block - window + 1 <= j_min / block  <=>  i <= i_w
                const int64_t i_w = (j_min / block + window) * (int64_t)block - 1;
                // (y0 + 31) / G <= i_w  <=>  y0 + 31 <= i_w * G + G - 1
                const int64_t hi_w = i_w * G + G - 32;
                if (hi_w < hi) hi = hi_w;
            }
            if (lo <= hi) { y_int_lo = (int)lo; y_int_hi = (int)(hi < 2147483647LL ? hi : 2147483647LL); }
        }
    }

    // From here on the two roles run separate instantiations of the same code (role 0: S = Y1 X1^T;
    // role 1: T = Y2 X2^T): each then has registers for its own operand fragments
    // and its own share of the accumulators, and no branch on the role sits inside the tile loop. The
    // workgroup barriers of the two instantiations pair up one to one.
    auto run = [&](auto role_c) {
    constexpr int ROLE = decltype(role_c)::value;
    // ---- the stationary side: matrix-core B operands in registers --------------------------------
    bf16x8 xf[ROLE == 0 ? DQK / 16 : DV / 16];
    constexpr int IN_AGPR = (256 - (ROLE == 0 ? C::ND0 : C::ND1) * 32) / 4;  // fragments that live in AGPRs
    const int64_t x_idx = (int64_t)xt * 64 + xb * 32 + ln;          // row (i * G + head) or key
    const int64_t x_c = x_idx < (KEYS ? S : R) ? x_idx : (KEYS ? S : R) - 1;
    int x_i = 0;                                                     // !KEYS: position of this lane's row
    float x_lse2 = 0.f, x_D = 0.f;
    {
        const uint16_t *xp;
        if (!KEYS) {
            const int64_t i = x_c / G;
            const int hh = (int)(x_c - i * G);
            x_i = (int)i;
            const int64_t qrow = (((int64_t)b * S + i) * p.Hq + (int64_t)g * G + hh);
            xp = ROLE == 0 ? p.q + qrow * DQK : p.dout + qrow * DV;
            const float2 st = p.rowstat[((int64_t)b * p.Hkv + g) * p.r_pad + x_c];
            x_lse2 = st.x;
            x_D = st.y;
        } else {
            const int64_t krow = ((int64_t)b * S + x_c) * p.Hkv + g;
            xp = ROLE == 0 ? p.k + krow * DQK : p.v + krow * (ALIAS ? DQK : DV);
        }
        xp += lh * 8;
#pragma unroll
        for (int kk = 0; kk < (ROLE == 0 ? DQK / 16 : DV / 16); ++kk) xf[kk] = *(const bf16x8 *)(xp + kk * 16);
        // Accumulators and fragments together exceed the 256 AGPRs. Left alone, the allocator treats the
        // fragments as vector registers it parks in AGPRs, and copies four registers back before every
        // matrix instruction; told which fragments live in AGPRs for good (a matrix instruction reads
        // them there) and which in VGPRs, it copies nothing.
#pragma unroll
        for (int kk = 0; kk < (ROLE == 0 ? DQK / 16 : DV / 16); ++kk) {
            if (kk < IN_AGPR) asm volatile("" : "+a"(xf[kk]));
            else asm volatile("" : "+v"(xf[kk]));
        }
    }
    const int w_lo_row = KEYS ? 0 : window_begin_of(x_i, window, block);
    int g_shift = 5;  // KEYS: log2(G) for G < 32, else 5
    if (G < 32) { g_shift = 0; while ((1 << g_shift) < G) ++g_shift; }

    // ---- global -> LDS copy plan of a streamed tile (the same for every tile) ---------------------
    // Instruction n fills LDS bytes [n*1024, n*1024 + 1024) of the stage: slot n*64 + lane of the
    // padded tile it belongs to is chunk (slot % CPR) of item (slot / CPR). The padding chunk of a row
    // and the slots past the tile fetch a valid chunk that nobody reads back; items past the end of
    // the tensor are cut to the last valid one by clamping the offset (offsets grow with the item).
    const int64_t pos_stride = KEYS ? (int64_t)p.Hq : (int64_t)p.Hkv;   // rows between consecutive positions
    auto item_offset = [&](int item, int width) -> uint32_t {           // byte offset of a tile item, row width in elements
        if (!KEYS) return (uint32_t)((int64_t)item * pos_stride * width * 2);
        if (G >= 32) return (uint32_t)(item * width * 2);               // 32 heads of one position
        return (uint32_t)(((int64_t)(item / G) * pos_stride + item % G) * width * 2);
    };
    constexpr int W2 = (!KEYS && ALIAS) ? DQK : DV;                      // element width of a Y2 row in memory
    // per-lane byte offset of this lane's 16 bytes within the global tile, for instruction n of a sub-tile
    auto lane_offset = [&](int kind, int n) -> uint32_t {
        if (kind == 3) return (lane < 15 ? lane : 15) * 16;  // 32 rows x 8 bytes of statistics
        const int cpr = kind == 1 ? C::CPR1 : C::CPR2;
        const int slot = n * 64 + lane, item = slot / cpr < 31 ? slot / cpr : 31;
        const int c = slot % cpr < cpr - 2 ? slot % cpr : cpr - 2;
        return item_offset(item, kind == 1 ? DQK : W2) + c * 16;
    };
    // the extra instruction of this wave (wave-uniform): 0 none, 1 / 2 instruction x_instr of the first /
    // second sub-tile, 3 the statistics
    int x_kind = 0, x_instr = 0;
    if (wave < C::R1) { x_kind = 1; x_instr = 4 * C::A1 + wave; }
    else if (wave < C::R1 + C::R2) { x_kind = 2; x_instr = 4 * C::A2 + (wave - C::R1); }
    else if (wave < C::NEXTRA) { x_kind = 3; }
    x_kind = __builtin_amdgcn_readfirstlane(x_kind);
    x_instr = __builtin_amdgcn_readfirstlane(x_instr);
    uint32_t yoff[C::PER_WAVE];
#pragma unroll
    for (int c = 0; c < C::A1; ++c) yoff[c] = lane_offset(1, c * 4 + wave);
#pragma unroll
    for (int c = 0; c < C::A2; ++c) yoff[C::A1 + c] = lane_offset(2, c * 4 + wave);
    yoff[C::A1 + C::A2] = x_kind ? lane_offset(x_kind, x_instr) : 0u;
    const char *y1_all = KEYS ? (const char *)p.q : (const char *)p.k;
    const char *y2_all = KEYS ? (const char *)p.dout : (const char *)p.v;
    // what the copy instructions of one tile share (all wave-uniform)
    struct TileCopy {
        const char *b1, *b2, *bx;         // global start of the tile's sub-tiles; of the extra instruction's
        uint32_t max1, max2, maxx;        // largest valid per-lane offset
        uint32_t dst1, dst2, dstx;        // LDS address of this wave's first chunk of a sub-tile; of its extra chunk
    };
    // (everything about a tile that does not depend on the tile is worked out here, once: the wave has
    // nothing else to issue while it computes addresses, so every instruction of the per-tile part
    // costs its full latency)
    const int n_y = (int)(KEYS ? R : S);                              // items on the streamed side (fits 32 bits)
    const int64_t row_base = KEYS ? (int64_t)b * S * p.Hq + (int64_t)g * G : (int64_t)b * S * p.Hkv + g;
    const int row_step = KEYS ? p.Hq - G : 0;                         // KEYS: tensor rows skipped per position
    const char *stat_base = (const char *)(p.rowstat + ((int64_t)b * p.Hkv + g) * p.r_pad);
    const uint32_t max1_full = item_offset(31, DQK) + (C::CPR1 - 2) * 16;
    const uint32_t max2_full = item_offset(31, W2) + (C::CPR2 - 2) * 16;
    const uint32_t dstx_off = (x_kind == 1 ? x_instr : x_kind == 2 ? C::N1 + x_instr : C::N1 + C::N2) * 1024;
    auto plan_tile = [&](int t, int stage) {
        const int y0 = y_tile(t) * 32;                               // first row / key of the tile
        // tensor row (of d elements) the tile starts at
        const int64_t row0 = KEYS ? row_base + y0 + (int64_t)div_g(y0) * row_step : row_base + (int64_t)y0 * p.Hkv;
        TileCopy tc;
        tc.b1 = y1_all + row0 * (DQK * 2);
        tc.b2 = y2_all + row0 * (W2 * 2);
        tc.max1 = max1_full;
        tc.max2 = max2_full;
        if (y0 + 31 >= n_y) {                                        // the ragged last tile: cut at its last valid item
            const int lim = n_y - 1 - y0;
            tc.max1 = item_offset(lim, DQK) + (C::CPR1 - 2) * 16;
            tc.max2 = item_offset(lim, W2) + (C::CPR2 - 2) * 16;
        }
        const uint32_t base = smem_lds + stage * C::STAGE;
        tc.dst1 = base + wave * 1024;
        tc.dst2 = base + C::OFF_Y2 + wave * 1024;
        tc.bx = x_kind == 1 ? tc.b1 : x_kind == 2 ? tc.b2 : stat_base + (int64_t)y0 * 8;
        tc.maxx = x_kind == 1 ? tc.max1 : x_kind == 2 ? tc.max2 : 0xffffffffu;
        tc.dstx = base + dstx_off;
        return tc;
    };
    // copy instruction c of this wave (c < PER_WAVE, a constant after unrolling)
    auto issue_one = [&](const TileCopy &tc, int c) {
        if (c < C::A1) copy_1k(tc.b1, yoff[c] < tc.max1 ? yoff[c] : tc.max1, tc.dst1 + c * 4096);
        else if (c < C::A1 + C::A2) copy_1k(tc.b2, yoff[c] < tc.max2 ? yoff[c] : tc.max2, tc.dst2 + (c - C::A1) * 4096);
        else if (x_kind) copy_1k(tc.bx, yoff[c] < tc.maxx ? yoff[c] : tc.maxx, tc.dstx);  // wave-uniform
    };

    constexpr int ND = ROLE == 0 ? C::ND0 : C::ND1;  // column blocks of this wave (each for both blocks of X)
    f32x16 acc[ND][2];
#pragma unroll
    for (int a = 0; a < ND; ++a)
#pragma unroll
        for (int x2 = 0; x2 < 2; ++x2)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][x2][e] = 0.f;
    // Which column blocks: the two waves of a role (xb = 0, 1) take alternate runs. With a shared
    // accumulator for dK and dV, blocks below d_v take both products; role 1's blocks are dealt so that
    // both of its waves get the same number of those (a < NDBL take two products, the rest one).
    constexpr int NDBL = (KEYS && !C::SPLIT_KV) ? (ROLE == 0 ? ND : C::NDBL1) : 0;
    auto col_block = [&](int a) {
        if (C::SPLIT_KV) return xb * ND + a;
        if (ROLE == 0) return xb * ND + a;
        if (!KEYS) return 2 * C::ND0 + xb * ND + a;
        return a < NDBL ? 2 * C::ND0 + xb * NDBL + a : DV / 32 + xb * (ND - NDBL) + (a - NDBL);
    };

    char *region = smem + C::OFF_BUF + xb * C::XREGION;   // dS rows of this block of X, then its p rows
    char *xch = smem + C::OFF_XCH + xb * C::XCH;          // T of this block of X, from its role-1 wave to its role-0 wave

    {
        const TileCopy tc0 = plan_tile(0, 0);
#pragma unroll
        for (int cu = 0; cu < C::PER_WAVE; ++cu) issue_one(tc0, cu);
    }
    // Everything requested from global memory so far (operand fragments, row statistics) is waited
    // for here, with a wait the compiler sees: left to its own bookkeeping it would wait for those
    // loads inside the loop, with counts that also drain the tile copies it does not know about.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    // The copy instructions of the next tile are issued one at a time between the matrix instructions
    // of phase 1 (in one burst they fill the memory pipeline's queue and the wave stalls on them for
    // longer than a phase takes), and none in phase 2: a copy requested that late is still on its way
    // when the next iteration waits for it (measured: 680 cycles per tile).
    constexpr int QD_OWN = ROLE == 0 ? 0 : 2, QD_GIVE = ROLE == 0 ? 2 : 0;
    // The four steps of a tile, strung together by the tile loop below.
    // Phase 1 on the tile in stage `st`, with this wave's copy instructions of plan `tc` woven in:
    auto phase1 = [&](const int st, const TileCopy &tc, f32x16 &c) {
        const char *tile = smem + st * C::STAGE;
        // ---- phase 1: one 32 x 32 block of S or T ---------------------------------------------------
        // S reads the first streamed tile; T the second when there is one (else the values are the key
        // rows' prefix)
        constexpr int A_OFF = (ROLE == 1 && C::HAS_Y2) ? C::OFF_Y2 : 0, A_ROW = (ROLE == 1 && C::HAS_Y2) ? C::ROW2 : C::ROW1;
        constexpr bool WIDE = (DQK == 576 && DV == 512);
        if constexpr (WIDE) {
            // Wide rows: the whole phase is one generated asm statement (score_asm.h), as the forward's
            // score phase is: fragment kk + 6 is fetched from LDS while fragment kk feeds the matrix core,
            // with the exact lgkmcnt each step needs, and this wave's copy instructions of the next tile
            // issue between the matrix instructions.
            static_assert(!WIDE || (C::A1 == 9 && C::A2 == (KEYS ? 8 : 0) && C::A2_WOVEN == (KEYS ? 2 : 0)), "one asm variant per copy plan");
            static_assert(!WIDE || IN_AGPR == (ROLE == 0 ? 32 : 24), "one asm variant per register split");
            bf16x8 kf[LOZA_SCORE_DEPTH_576];
            uint32_t tmp;
            const uint32_t a_addr = smem_lds + st * C::STAGE + A_OFF + ln * A_ROW + lh * 16;
            if constexpr (KEYS) {
                if constexpr (ROLE == 0) LOZA_BWD_PHASE1_K36_A9_B2_G32(c, kf, tmp, a_addr, xf, yoff, tc, wave, C::NEXTRA);
                else LOZA_BWD_PHASE1_K32_A9_B2_G24(c, kf, tmp, a_addr, xf, yoff, tc, wave, C::NEXTRA);
            } else {
                if constexpr (ROLE == 0) LOZA_BWD_PHASE1_K36_A9_B0_G32(c, kf, tmp, a_addr, xf, yoff, tc, wave, C::NEXTRA);
                else LOZA_BWD_PHASE1_K32_A9_B0_G24(c, kf, tmp, a_addr, xf, yoff, tc, wave, C::NEXTRA);
            }
        } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) c[e] = 0.f;
        // (fragments of the streamed tile are fetched PF steps ahead of the matrix instruction that
        // uses them; the scheduling barriers keep the compiler from hoisting all of them to the top,
        // which costs registers it then finds by spilling -- and a reload from scratch waits for every
        // vector-memory operation in flight, the copy of the next tile included)
        {
            constexpr int NS = ROLE == 0 ? DQK / 16 : DV / 16, PF = 8, EVERY = NS / C::PER_WAVE > 0 ? NS / C::PER_WAVE : 1;
            const char *ya = tile + A_OFF + ln * A_ROW + lh * 16;
            bf16x8 af[PF];
#pragma unroll
            for (int d = 0; d < PF; ++d) af[d] = *(const bf16x8 *)(ya + d * 32);
#pragma unroll
            for (int kk = 0; kk < NS; ++kk) {
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk % PF], xf[kk], c, 0, 0, 0);
                if (kk + PF < NS) af[kk % PF] = *(const bf16x8 *)(ya + (kk + PF) * 32);
                if (kk % EVERY == 0 && kk / EVERY < C::PER_WAVE) issue_one(tc, kk / EVERY);
                __builtin_amdgcn_sched_barrier(0);
            }
            // (copies that did not find a slot above)
#pragma unroll
            for (int cu = (NS + EVERY - 1) / EVERY; cu < C::PER_WAVE; ++cu) issue_one(tc, cu);
        }
        }
    };
    auto hand_over = [&](const f32x16 &c) {
        // The elementwise step is shared: of this lane's four runs of four values, the S wave processes
        // runs 0, 1 and the T wave runs 2, 3; each hands the other the half of its block it does not
        // process itself (xch: [role of the writer][run][lane] x 16 bytes).
#pragma unroll
        for (int q2 = 0; q2 < 2; ++q2) {
            const int qd = QD_GIVE + q2;
            float4 w;
            w.x = c[4 * qd]; w.y = c[4 * qd + 1]; w.z = c[4 * qd + 2]; w.w = c[4 * qd + 3];
            *(float4 *)(xch + ((ROLE * 2 + q2) * 64 + lane) * 16) = w;
        }
    };
    // (tile `t_idx` of this work item, in stage `st`)
    auto elementwise_step = [&](const f32x16 &c, const int t_idx, const int st, const TileCopy &tc) {
        const char *tile = smem + st * C::STAGE;
        // ---- elementwise: p = exp2(scale log2e s - lse log2e), dS = scale p (T - D), masked ----------
        // four values at a time: this lane's 16 values are four runs of four consecutive y, and a run
        // is one 8-byte store into the [x][y] buffers (y contiguous)
        {
            const int y0 = y_tile(t_idx) * 32;
            char *ps = region + ln * C::PROW + (4 * lh) * 2;
            const float2 *stat = (const float2 *)(tile + C::OFF_STAT);
            bool interior;
            if (!KEYS) {
                // lane = query row, values = keys y0 + 8 qd + 4 lh + t
                interior = (y0 + 31 <= i_min) && ((y0 + 31 < n_sink) || (y0 >= w_lo_max));
            } else {
                // lane = key, values = query rows y0 + 8 qd + 4 lh + t
                interior = y0 >= y_int_lo && y0 <= y_int_hi;
            }
            // KEYS: position of row y0 + y is i_tile + (y >> g_shift): a tile is 32 / G whole positions
            // (G a power of two) or part of one position (G a multiple of 32: the shift drops every y)
            // (one branch for the whole tile: interior tiles, nearly all of them, evaluate no predicate)
            auto elementwise = [&](auto masked) {
            constexpr bool MASKED = decltype(masked)::value;
            int i_tile = 0, w_lo_tile = 0;
            if constexpr (MASKED && KEYS) {
                i_tile = div_g(y0);
                w_lo_tile = window_begin_of(i_tile, window, block);
            }
            // (everything this step reads from LDS is requested before the first result is written back:
            // a read behind a write would wait for it, and the wave has nothing to hide that behind)
            // (the copy instructions of the second sub-tile that phase 1 left out: two now, two after each half)
            constexpr int LATE = C::A2 - C::A2_WOVEN, LATE_STEP = (LATE + 2) / 3;
            auto late_copies = [&](int part) {
#pragma unroll
                for (int cc = part * LATE_STEP; cc < (part + 1) * LATE_STEP; ++cc)
                    if (cc < LATE) issue_one(tc, C::A1 + C::A2_WOVEN + cc);
            };
            late_copies(0);
            float4 o4[2];
            float2 sd[2][4];
#pragma unroll
            for (int q2 = 0; q2 < 2; ++q2) {
                o4[q2] = *(const float4 *)(xch + (((1 - ROLE) * 2 + q2) * 64 + lane) * 16);
                if (KEYS) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) sd[q2][t] = stat[8 * (QD_OWN + q2) + 4 * lh + t];
                }
            }
#pragma unroll
            for (int q2 = 0; q2 < 2; ++q2) {
                const int qd = QD_OWN + q2;
                const float other[4] = {o4[q2].x, o4[q2].y, o4[q2].z, o4[q2].w};   // the other wave's block: T for the S wave, S for the T wave
                float pv[4], dsv[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int e = 4 * qd + t, y = 8 * qd + 4 * lh + t;
                    float lse2, D;
                    bool ok = true;
                    if (!KEYS) {
                        lse2 = x_lse2; D = x_D;
                        const int j = y0 + y;
                        if (MASKED) ok = (j <= x_i) & ((j < n_sink) | (j >= w_lo_row));
                    } else {
                        lse2 = sd[q2][t].x; D = sd[q2][t].y;
                        if (MASKED) {
                            const int i = i_tile + (y >> g_shift), j = (int)x_idx;
                            const int w_lo = G >= 32 ? w_lo_tile : window_begin_of(i, window, block);
                            ok = (y0 + y < (int)R) & (j < (int)S) & (j <= i) & ((j < n_sink) | (j >= w_lo));
                        }
                    }
                    const float sv = ROLE == 0 ? c[e] : other[t], tv = ROLE == 0 ? other[t] : c[e];
                    const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sv, p.scale_log2, -lse2));
                    pv[t] = ok ? pe : 0.f;
                    dsv[t] = ok ? p.scale * pe * (tv - D) : 0.f;
                }
                late_copies(1 + q2);
                u32x2 w;
                w[0] = pack_bf16(dsv[0], dsv[1]);
                w[1] = pack_bf16(dsv[2], dsv[3]);
                *(u32x2 *)(ps + qd * 16) = w;
                if (KEYS) {
                    w[0] = pack_bf16(pv[0], pv[1]);
                    w[1] = pack_bf16(pv[2], pv[3]);
                    *(u32x2 *)(ps + 32 * C::PROW + qd * 16) = w;
                }
            }
            };
            if (interior) elementwise(std::false_type{});
            else elementwise(std::true_type{});
        }
    };
    auto phase2 = [&](const int st) {
        const char *tile = smem + st * C::STAGE;
        // ---- phase 2: Acc^T[column block][x] += Y^T dS (+ Y2^T p), both blocks of X per fragment -------
        {
            const char *b0 = smem + C::OFF_BUF + ln * C::PROW + lh * 16;   // dS rows of block 0 of X ([x][y])
            const char *t1 = tile, *t2 = tile + C::OFF_Y2;
            // The fragments of this wave as a flat list of (key step, column block, product); product 1
            // (Y2^T p, the dV part of a shared accumulator) exists for the first NDBL blocks. Fetched PF
            // entries ahead; every fragment feeds one matrix instruction per block of X.
            constexpr int PER_KS = ND + NDBL;
            constexpr int NF = 2 * PER_KS, PF = 4;
            auto entry = [](int m, int &ks, int &a, int &prod) {
                ks = m / PER_KS;
                const int r = m % PER_KS;
                if (r < 2 * NDBL) { a = r / 2; prod = r % 2; } else { a = r - NDBL; prod = 0; }
            };
            auto frag = [&](int m) {
                int ks, a, prod;
                entry(m, ks, a, prod);
                const bool second = C::SPLIT_KV ? ROLE == 1 : prod == 1;
                return second ? read_transposed(t2, C::ROW2, col_block(a), ks, lane) : read_transposed(t1, C::ROW1, col_block(a), ks, lane);
            };
            bf16x8 b_ds[2], b_p[2];
            auto load_b = [&](int ks) {
#pragma unroll
                for (int x2 = 0; x2 < 2; ++x2) {
                    b_ds[x2] = *(const bf16x8 *)(b0 + x2 * C::XREGION + ks * 32);
                    b_p[x2] = KEYS ? *(const bf16x8 *)(b0 + x2 * C::XREGION + 32 * C::PROW + ks * 32) : b_ds[x2];
                }
            };
            load_b(0);
            bf16x8 fr[PF];
#pragma unroll
            for (int m = 0; m < PF && m < NF; ++m) fr[m] = frag(m);
#pragma unroll
            for (int m = 0; m < NF; ++m) {
                int ks, a, prod;
                entry(m, ks, a, prod);
                const bool use_p = C::SPLIT_KV ? ROLE == 1 : prod == 1;
                const bf16x8 f = fr[m % PF];
                acc[a][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, use_p ? b_p[0] : b_ds[0], acc[a][0], 0, 0, 0);
                acc[a][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, use_p ? b_p[1] : b_ds[1], acc[a][1], 0, 0, 0);
                if (m + PF < NF) fr[m % PF] = frag(m + PF);
                if (m == PER_KS - 1) load_b(1);  // the second key step's dS and p
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Two stages, three barriers per tile: (A) tile u has landed and tile u - 1 is no longer read,
    // (B) the halves of S and T are handed over, (C) dS and p are complete. (A third stage fits the dQ
    // kernel and lets phase 2 of a tile follow phase 1 of the next without barrier A: built, 0.4 %.)
    for (int u = 0; u < nt; ++u) {
        const int st = u & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's copies of tile u have landed ...
        __syncthreads();                                  // ... everyone's; tile u - 1 is no longer read
        const TileCopy tc = plan_tile(u + 1 < nt ? u + 1 : u, st ^ 1);
        f32x16 c;
        phase1(st, tc, c);
        hand_over(c);
        __syncthreads();
        elementwise_step(c, u, st, tc);
        __syncthreads();
        phase2(st);
    }

    // (the last iteration copied its own tile once more rather than branch around every copy
    // instruction; nothing may still be on its way into LDS when the workgroup ends)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // ---- epilogue: lane = item of X, 16 values of a block = four runs of four consecutive columns ------
#pragma unroll
    for (int x2 = 0; x2 < 2; ++x2) {
        const int64_t xi = (int64_t)xt * 64 + x2 * 32 + ln;
        if (xi >= (KEYS ? S : R)) continue;
        if (!KEYS) {
            const int64_t i = xi / G;
            const int hh = (int)(xi - i * G);
            uint16_t *op = p.dq + (((int64_t)b * S + i) * p.Hq + (int64_t)g * G + hh) * DQK + 4 * lh;
#pragma unroll
            for (int a = 0; a < ND; ++a)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    u32x2 w;
                    w[0] = pack_bf16(acc[a][x2][4 * qd], acc[a][x2][4 * qd + 1]);
                    w[1] = pack_bf16(acc[a][x2][4 * qd + 2], acc[a][x2][4 * qd + 3]);
                    *(u32x2 *)(op + col_block(a) * 32 + qd * 8) = w;
                }
        } else if (partial) {
            // row [dK (d_qk) | dV (d_v, separate values only)] of fp32 partial sums
            constexpr int COLS = C::SPLIT_KV ? DQK + DV : DQK;
            float *op = p.part + ((((int64_t)b * p.Hkv + g) * p.n_sink_kt + xt) * p.max_chunks + chunk) * 64 * COLS +
                        (int64_t)(x2 * 32 + ln) * COLS + ((C::SPLIT_KV && ROLE == 1) ? DQK : 0) + 4 * lh;
#pragma unroll
            for (int a = 0; a < ND; ++a)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    float4 w;
                    w.x = acc[a][x2][4 * qd]; w.y = acc[a][x2][4 * qd + 1]; w.z = acc[a][x2][4 * qd + 2]; w.w = acc[a][x2][4 * qd + 3];
                    *(float4 *)(op + col_block(a) * 32 + qd * 8) = w;
                }
        } else {
            const int64_t krow = ((int64_t)b * S + xi) * p.Hkv + g;
            uint16_t *op = ((C::SPLIT_KV && ROLE == 1) ? p.dv + krow * DV : p.dk + krow * DQK) + 4 * lh;
#pragma unroll
            for (int a = 0; a < ND; ++a)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    u32x2 w;
                    w[0] = pack_bf16(acc[a][x2][4 * qd], acc[a][x2][4 * qd + 1]);
                    w[1] = pack_bf16(acc[a][x2][4 * qd + 2], acc[a][x2][4 * qd + 3]);
                    *(u32x2 *)(op + col_block(a) * 32 + qd * 8) = w;
                }
        }
    }
    };
    if (role == 0) run(std::integral_constant<int, 0>{});
    else run(std::integral_constant<int, 1>{});
}

// Sum of the chunk partials of the key tiles that hold sink keys, in chunk order, rounded once.
// One thread per four columns of one key.
template <int DQK, int DV, bool ALIAS>
__global__ __launch_bounds__(256) void ssa_bwd_reduce_kernel(const BwdParams p)
{
    constexpr int COLS = ALIAS ? DQK : DQK + DV;
    constexpr int TPK = COLS / 4;  // threads per key
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n_keys = (int64_t)p.B * p.Hkv * p.n_sink_kt * 64;
    if (t >= n_keys * TPK) return;
    const int c = (int)(t % TPK) * 4;
    const int64_t key = t / TPK;
    const int x = (int)(key % 64);
    const int64_t tile = key / 64;  // flat (b, g, kt)
    const int kt = (int)(tile % p.n_sink_kt);
    const int64_t bg = tile / p.n_sink_kt;
    const int g = (int)(bg % p.Hkv);
    const int64_t b = bg / p.Hkv;
    const int64_t j = (int64_t)kt * 64 + x;
    if (j >= p.S) return;
    int yt_lo, yt_hi;
    bwd_key_tile_rows(p, kt, yt_lo, yt_hi);
    const int chunks = (yt_hi - yt_lo + 1 + p.chunk_tiles - 1) / p.chunk_tiles;
    float4 s = {0.f, 0.f, 0.f, 0.f};
    const float *pp = p.part + (tile * p.max_chunks * 64 + x) * COLS + c;
    for (int ch = 0; ch < chunks; ++ch) {
        const float4 v = *(const float4 *)(pp + (int64_t)ch * 64 * COLS);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    u32x2 w;
    w[0] = pack_bf16(s.x, s.y);
    w[1] = pack_bf16(s.z, s.w);
    const int64_t krow = (b * p.S + j) * p.Hkv + g;
    if (c < DQK) *(u32x2 *)(p.dk + krow * DQK + c) = w;
    else *(u32x2 *)(p.dv + krow * DV + (c - DQK)) = w;
}

template <int DQK, int DV, bool ALIAS>
static hipError_t launch_backward_t(const BwdParams &p, hipStream_t stream)
{
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq;
    hipLaunchKernelGGL((ssa_bwd_rowstat_kernel<DV>), dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    {
        using C = BwdCfg<DQK, DV, ALIAS, false>;
        auto kern = ssa_bwd_kernel<DQK, DV, ALIAS, false>;
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        const int64_t blocks = ((p.S * p.G + 63) / 64) * p.Hkv * p.B;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    {
        using C = BwdCfg<DQK, DV, ALIAS, true>;
        auto kern = ssa_bwd_kernel<DQK, DV, ALIAS, true>;
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        const int64_t n_kt = (p.S + 63) / 64;
        const int64_t blocks = ((int64_t)p.n_sink_kt * p.max_chunks + (n_kt - p.n_sink_kt)) * p.Hkv * p.B;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (p.n_sink_kt > 0 && p.max_chunks > 1) {
        constexpr int COLS = ALIAS ? DQK : DQK + DV;
        const int64_t threads = (int64_t)p.B * p.Hkv * p.n_sink_kt * 64 * (COLS / 4);
        hipLaunchKernelGGL((ssa_bwd_reduce_kernel<DQK, DV, ALIAS>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

// The row tiles of the key-stationary kernel must not straddle positions unevenly: heads per group a
// power of two up to 32 (a tile is 32 / G whole positions) or a multiple of 32 (a tile is part of one).
bool bwd_group_supported(int G) { return G >= 1 && (G % 32 == 0 || (G < 32 && (G & (G - 1)) == 0)); }

hipError_t launch_backward_bf16(const BwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream)
{
    if (d_qk == 576 && d_v == 512 && alias) return launch_backward_t<576, 512, true>(p, stream);
    if (d_qk == 128 && d_v == 128) return alias ? launch_backward_t<128, 128, true>(p, stream)
                                                : launch_backward_t<128, 128, false>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace loza
