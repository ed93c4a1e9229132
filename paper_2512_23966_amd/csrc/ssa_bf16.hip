// bf16 streaming-sparse-attention kernels for gfx950 (MI355X): prefill and split-key decode.
//
// What is computed: O* = softmax(scale * Q K*^T) V* over the live key set of every query
// (paper: Architecture section, Eq. 2 / Eq. 4; with window >= S this is Eq. 1), plus the natural
// log of the softmax denominator.  live(i) = { j <= i : j < n_sink or i - j < window }.
//
// How it is mapped to the machine (one workgroup = 4 wavefronts = 1 per SIMD):
//   * Rows of a workgroup tile are (position, head-in-group) pairs of ONE key/value head, so all
//     query heads that share a latent (absorbed MLA) reuse each key tile from a single LDS copy.
//   * Only live key tiles are enumerated: the sink tiles, then the window tiles, by closed-form
//     integer arithmetic (no schedule metadata in memory, the same schedule for every head).
//     Interior tiles take no mask; only tiles cut by the causal diagonal, the window's trailing
//     edge or the sink edge evaluate the predicate per element.
//   * Score phase: wave (wr, wk) holds the 32 query rows of row block wr in registers as MFMA B
//     operands and computes S^T = K Q^T for key block wk of the tile (32x32x16 bf16 MFMA), so that
//     one lane owns one query row and the online-softmax statistics need a single cross-lane step.
//   * P is rounded to bf16 and handed over through LDS; in the value phase wave w owns the
//     d_v / 4 output columns [w*d_v/4, (w+1)*d_v/4) of ALL rows of the tile, so each value
//     fragment (read transposed from the key tile with ds_read_b64_tr_b16) is fetched once per
//     workgroup instead of once per wave.
//   * Key tiles stream HBM/L2 -> LDS with global_load_lds_dwordx4 (no register staging), double
//     buffered; LDS rows are padded by 16 bytes so 128-bit fragment reads are bank-conflict free.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ssa_kernels.h"

namespace loza {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef __attribute__((address_space(1))) const void *glb_void_ptr;

#define LOZA_NEG_INF (-__builtin_inff())

static __device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 v;
    v[0] = (__bf16)a;  // round to nearest even
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

// Workgroup barrier that orders LDS traffic only: in-flight global -> LDS tile copies of the
// NEXT tile stay in flight across it (a barrier with a full memory fence would drain them).
static __device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

static __device__ __forceinline__ float xor32(float x)
{
    // value held by the lane in the other half of the wavefront (lane ^ 32)
    return __shfl_xor(x, 32, 64);
}

template <int DQK, int DV, int RB, int KB, bool ALIAS>
struct TileCfg {
    static constexpr int M = 32 * RB;            // query rows per workgroup
    static constexpr int N = 32 * KB;            // keys per tile
    static constexpr int NW = RB * KB;           // wavefronts
    static_assert(NW == 4, "four wavefronts, one per SIMD");
    static constexpr int DVW = DV / NW;          // output columns owned by one wave (value phase)
    static constexpr int DVB = DVW / 32;         // 32-column blocks of them
    static_assert(DVB * 32 * NW == DV, "d_v must be a multiple of 128");
    static_assert(DQK % 16 == 0, "d_qk must be a multiple of 16");
    static constexpr int KROW = DQK * 2 + 16;    // LDS bytes per key row (16 bytes of padding)
    static constexpr int VROW = ALIAS ? KROW : DV * 2 + 16;
    static constexpr int KCPR = KROW / 16;       // 16-byte chunks per padded key row
    static constexpr int VCPR = VROW / 16;
    static constexpr int KTILE = N * KROW;
    static constexpr int VTILE = ALIAS ? 0 : N * VROW;
    static constexpr int STAGE = KTILE + VTILE;
    static constexpr int NSTAGE = 2;
    static constexpr int PROW = N * 2 + 16;      // LDS bytes per row of P (padded)
    static constexpr int OFF_P = NSTAGE * STAGE;
    static constexpr int OFF_ALPHA = OFF_P + M * PROW;        // float[M]
    static constexpr int OFF_FLAG = OFF_ALPHA + M * 4;        // int[RB] (padded to 16)
    static constexpr int OFF_SMAX = OFF_FLAG + 16;            // float[KB][M]
    static constexpr int OFF_LPART = OFF_SMAX + KB * M * 4;   // float[KB][M]
    static constexpr int LDS_BYTES = OFF_LPART + KB * M * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit the 160 KB LDS");
    // global -> LDS copy: one instruction moves 64 consecutive 16-byte chunks of the padded tile
    static constexpr int K_INSTR = (N * KCPR + 63) / 64;
    static constexpr int V_INSTR = ALIAS ? 0 : (N * VCPR + 63) / 64;
    static constexpr int K_PER_WAVE = (K_INSTR + NW - 1) / NW;
    static constexpr int V_PER_WAVE = (V_INSTR + NW - 1) / NW;
};

// One lane's share of one copy instruction: (row in tile, chunk in row) or "idle".
static __device__ __forceinline__ int chunk_code(int instr, int n_instr, int lane, int rows, int cpr)
{
    if (instr >= n_instr) return -1;
    const int p = instr * 64 + lane;
    if (p >= rows * cpr) return -1;
    const int row = p / cpr, c = p - row * cpr;
    if (c == cpr - 1) return -1;  // the padding chunk of a row
    return row | (c << 8);
}

template <int DQK, int DV, int RB, int KB, bool ALIAS, bool DECODE>
__global__ __launch_bounds__(256) void ssa_fwd_kernel(const FwdParams p)
{
    using C = TileCfg<DQK, DV, RB, KB, ALIAS>;
    constexpr int M = C::M, N = C::N;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
    const int wr = wave / KB, wk = wave % KB;

    // ---- which tile of which (batch, kv head) ------------------------------------------------
    int id = blockIdx.x;
    int split = 0;
    if (DECODE) { split = id % p.n_splits; id /= p.n_splits; }
    const int rt = p.row_tiles - 1 - (id % p.row_tiles);  // heaviest (latest) row tiles first
    id /= p.row_tiles;
    const int g = id % p.Hkv;
    const int b = id / p.Hkv;
    const int G = p.G;

    // valid key rows (a decode length beyond the cache is cut to the cache)
    const int64_t L = DECODE ? ((int64_t)p.seqlens[b] < p.S ? (int64_t)p.seqlens[b] : p.S) : p.S;
    const int64_t R = DECODE ? (int64_t)G : p.S * (int64_t)G;    // query rows of this (b, g)
    const int64_t r0 = (int64_t)rt * M;
    const int n_sink = p.n_sink, window = p.window;

    // ---- decode of an empty cache: a neutral partial ------------------------------------------
    if (DECODE && L <= 0) {
        for (int r = tid; r < M; r += 256) {
            if (r0 + r >= R) continue;
            const int64_t h = (int64_t)b * p.Hq + (int64_t)g * G + r0 + r;
            float *po = p.part_o + (h * p.n_splits + split) * DV;
            for (int c = 0; c < DV; ++c) po[c] = 0.f;
            p.part_ml[(h * p.n_splits + split) * 2 + 0] = LOZA_NEG_INF;
            p.part_ml[(h * p.n_splits + split) * 2 + 1] = 0.f;
        }
        return;
    }

    // ---- the query row this lane scores ---------------------------------------------------------
    const int64_t my_row = r0 + wr * 32 + ln;
    const int64_t my_row_c = my_row < R ? my_row : R - 1;
    const int i_row = DECODE ? (int)(L - 1) : (int)(my_row_c / G);
    const int i_min = DECODE ? (int)(L - 1) : (int)(r0 / G);
    const int i_max = DECODE ? (int)(L - 1) : (int)(((r0 + M - 1 < R) ? r0 + M - 1 : R - 1) / G);

    bf16x8 qf[DQK / 16];
    {
        const int hh = DECODE ? (int)my_row_c : (int)(my_row_c - (int64_t)i_row * G);
        const int64_t qrow = DECODE ? ((int64_t)b * p.Hq + (int64_t)g * G + hh)
                                    : (((int64_t)b * p.S + i_row) * p.Hq + (int64_t)g * G + hh);
        const uint16_t *qp = p.q + qrow * DQK + lh * 8;
#pragma unroll
        for (int kk = 0; kk < DQK / 16; ++kk) qf[kk] = *(const bf16x8 *)(qp + kk * 16);
    }

    // ---- live key tiles: sink tiles [0, nA), then window tiles [wt0, wt0 + nB) -------------------
    const int sink_end = n_sink < i_max + 1 ? n_sink : i_max + 1;
    const int win_begin = window > i_min ? 0 : i_min - window + 1;
    int nA = (sink_end + N - 1) / N;
    const int wt0 = win_begin / N, wt1 = i_max / N;
    int nB;
    if (wt0 <= nA) { nA = wt1 + 1; nB = 0; } else { nB = wt1 - wt0 + 1; }
    const int n_tiles = nA + nB;
    int t_begin = 0, t_end = n_tiles;
    if (DECODE) {
        const int per = (n_tiles + p.n_splits - 1) / p.n_splits;
        t_begin = split * per;
        t_end = t_begin + per < n_tiles ? t_begin + per : n_tiles;
    }

    // ---- global -> LDS copy plan of this lane (the same for every tile) --------------------------
    int kcode[C::K_PER_WAVE];
#pragma unroll
    for (int u = 0; u < C::K_PER_WAVE; ++u) kcode[u] = chunk_code(u * 4 + wave, C::K_INSTR, lane, N, C::KCPR);
    int vcode[C::V_PER_WAVE > 0 ? C::V_PER_WAVE : 1];
#pragma unroll
    for (int u = 0; u < C::V_PER_WAVE; ++u) vcode[u] = chunk_code(u * 4 + wave, C::V_INSTR, lane, N, C::VCPR);

    const int64_t kv_pos_stride_k = (int64_t)p.Hkv * DQK * 2;  // bytes between consecutive positions
    const int64_t kv_pos_stride_v = (int64_t)p.Hkv * DV * 2;
    const char *kbase = (const char *)p.k + ((int64_t)b * p.S * p.Hkv + g) * (int64_t)DQK * 2;
    const char *vbase = (const char *)p.v + ((int64_t)b * p.S * p.Hkv + g) * (int64_t)DV * 2;

    auto issue_tile = [&](int t, int stage) {
        const int kt = t < nA ? t : wt0 + (t - nA);
        const int64_t j0 = (int64_t)kt * N;
        const int lim = (L - 1 - j0) < (N - 1) ? (int)(L - 1 - j0) : N - 1;  // last valid row in tile
        const char *ksrc = kbase + j0 * kv_pos_stride_k;
        char *kdst = smem + stage * C::STAGE;
#pragma unroll
        for (int u = 0; u < C::K_PER_WAVE; ++u) {
            if (kcode[u] >= 0) {
                int row = kcode[u] & 0xff;
                row = row < lim ? row : lim;  // rows past the sequence end repeat its last row
                const int64_t off = (int64_t)row * kv_pos_stride_k + (kcode[u] >> 8) * 16;
                __builtin_amdgcn_global_load_lds((glb_void_ptr)(ksrc + off),
                                                 (lds_void_ptr)(kdst + (u * 4 + wave) * 1024), 16, 0, 0);
            }
        }
        if (!ALIAS) {
            const char *vsrc = vbase + j0 * kv_pos_stride_v;
            char *vdst = smem + stage * C::STAGE + C::KTILE;
#pragma unroll
            for (int u = 0; u < C::V_PER_WAVE; ++u) {
                if (vcode[u] >= 0) {
                    int row = vcode[u] & 0xff;
                    row = row < lim ? row : lim;
                    const int64_t off = (int64_t)row * kv_pos_stride_v + (vcode[u] >> 8) * 16;
                    __builtin_amdgcn_global_load_lds((glb_void_ptr)(vsrc + off),
                                                     (lds_void_ptr)(vdst + (u * 4 + wave) * 1024), 16, 0, 0);
                }
            }
        }
    };

    f32x16 o[C::DVB][RB];
#pragma unroll
    for (int db = 0; db < C::DVB; ++db)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][rb][e] = 0.f;
    float m_run = LOZA_NEG_INF;  // running row maximum of scale*log2(e)*q.k
    float l_run = 0.f;           // this lane's share of the running row sum

    float *s_alpha = (float *)(smem + C::OFF_ALPHA);
    int *s_flag = (int *)(smem + C::OFF_FLAG);
    float *s_smax = (float *)(smem + C::OFF_SMAX);
    float *s_lpart = (float *)(smem + C::OFF_LPART);
    char *s_p = smem + C::OFF_P;

    if (t_begin < t_end) issue_tile(t_begin, 0);

    for (int t = t_begin; t < t_end; ++t) {
        const int stage = (t - t_begin) & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of tile t has landed
        lds_barrier();                     // ... and everyone's; the other stage and P are free
        if (t + 1 < t_end) issue_tile(t + 1, stage ^ 1);

        const int kt = t < nA ? t : wt0 + (t - nA);
        const int j0 = kt * N;
        const char *ktile = smem + stage * C::STAGE;
        const char *vtile = ALIAS ? ktile : ktile + C::KTILE;

        // ---- scores: S^T[32 keys of block wk][32 rows of block wr] ----------------------------
        f32x16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = 0.f;
        {
            const char *kp = ktile + (wk * 32 + ln) * C::KROW + lh * 16;
#pragma unroll
            for (int kk = 0; kk < DQK / 16; ++kk) {
                const bf16x8 a = *(const bf16x8 *)(kp + kk * 32);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s, 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] *= p.scale_log2;

        // ---- mask, on tiles the pattern cuts ----------------------------------------------------
        const bool interior = (j0 + N - 1 <= i_min) && ((j0 + N - 1 < n_sink) || (i_max - j0 < window));
        if (!interior) {
            const int jb = j0 + wk * 32 + 4 * lh;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int j = jb + 8 * (e >> 2) + (e & 3);
                const bool ok = (j <= i_row) && (j < n_sink || i_row - j < window);
                s[e] = ok ? s[e] : LOZA_NEG_INF;
            }
        }

        // ---- online softmax ----------------------------------------------------------------------
        float mx = s[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s[e]);
        mx = fmaxf(mx, xor32(mx));
        if (KB > 1) {
            if (lh == 0) s_smax[wk * M + wr * 32 + ln] = mx;
            lds_barrier();
#pragma unroll
            for (int c = 0; c < KB; ++c) mx = fmaxf(mx, s_smax[c * M + wr * 32 + ln]);
        }
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == LOZA_NEG_INF) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s[e] = __builtin_amdgcn_exp2f(s[e] - m_use);
            psum += s[e];
        }
        l_run = l_run * alpha + psum;
        const bool rescale = __any(alpha != 1.0f);
        if (wk == 0) {
            if (lane == 0) s_flag[wr] = rescale ? 1 : 0;
            if (rescale && lh == 0) s_alpha[wr * 32 + ln] = alpha;
        }
        {
            char *pp = s_p + (wr * 32 + ln) * C::PROW + (wk * 32 + 4 * lh) * 2;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                u32x2 w;
                w[0] = pack_bf16(s[4 * qd + 0], s[4 * qd + 1]);
                w[1] = pack_bf16(s[4 * qd + 2], s[4 * qd + 3]);
                *(u32x2 *)(pp + qd * 16) = w;
            }
        }
        lds_barrier();

        // ---- values: O^T[d_v slice of this wave][all rows] += V^T P^T ------------------------------
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (__builtin_amdgcn_readfirstlane(s_flag[rb])) {
                const float a = s_alpha[rb * 32 + ln];
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
        {
            const int s16 = lane & 15, g16 = (lane >> 4) & 1;
            const char *vp = vtile + (lh * 8 + (s16 >> 2)) * C::VROW + (wave * C::DVW + g16 * 16 + (s16 & 3) * 4) * 2;
            const char *pb = s_p + ln * C::PROW + lh * 16;
#pragma unroll
            for (int ks = 0; ks < N / 16; ++ks) {
                bf16x8 pf[RB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) pf[rb] = *(const bf16x8 *)(pb + rb * 32 * C::PROW + ks * 32);
#pragma unroll
                for (int db = 0; db < C::DVB; ++db) {
                    const char *va = vp + ks * 16 * C::VROW + db * 64;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(va));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(va + 4 * C::VROW));
                    s16x8 a8;
                    a8[0] = lo[0]; a8[1] = lo[1]; a8[2] = lo[2]; a8[3] = lo[3];
                    a8[4] = hi[0]; a8[5] = hi[1]; a8[6] = hi[2]; a8[7] = hi[3];
                    const bf16x8 a = __builtin_bit_cast(bf16x8, a8);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb], o[db][rb], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue ----------------------------------------------------------------------------------
    {
        const float l_lane = l_run + xor32(l_run);
        if (lh == 0) s_lpart[wk * M + wr * 32 + ln] = l_lane;
    }
    lds_barrier();
    float l_tot_mine = 0.f;
#pragma unroll
    for (int c = 0; c < KB; ++c) l_tot_mine += s_lpart[c * M + wr * 32 + ln];

    if (!DECODE) {
        // lse = ln(sum_j exp(scale q.k_j)) = (m + log2 l) * ln 2
        if (wk == 0 && lh == 0 && my_row < R) {
            const int hh = (int)(my_row - (int64_t)i_row * G);
            p.lse[((int64_t)b * p.Hq + (int64_t)g * G + hh) * p.S + i_row] =
                (m_run + __builtin_amdgcn_logf(l_tot_mine)) * 0.69314718055994530942f;
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int64_t row = r0 + rb * 32 + ln;
            float l_tot = 0.f;
#pragma unroll
            for (int c = 0; c < KB; ++c) l_tot += s_lpart[c * M + rb * 32 + ln];
            const float inv = 1.0f / l_tot;
            if (row < R) {
                const int64_t i = row / G;
                const int hh = (int)(row - i * G);
                uint16_t *op = p.out + ((((int64_t)b * p.S + i) * p.Hq + (int64_t)g * G + hh) * DV) + wave * C::DVW + 4 * lh;
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
    } else {
        // partial result of this key split: unnormalised O (relative to m), m, l
        if (wk == 0 && lh == 0 && my_row < R) {
            const int64_t h = (int64_t)b * p.Hq + (int64_t)g * G + my_row;
            p.part_ml[(h * p.n_splits + split) * 2 + 0] = m_run;
            p.part_ml[(h * p.n_splits + split) * 2 + 1] = l_tot_mine;
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int64_t row = r0 + rb * 32 + ln;
            if (row < R) {
                const int64_t h = (int64_t)b * p.Hq + (int64_t)g * G + row;
                float *op = p.part_o + (h * p.n_splits + split) * DV + wave * C::DVW + 4 * lh;
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
}

// Merge of the key splits of one decode query (log-sum-exp rule, fixed split order):
//   m* = max_s m_s ;  w_s = 2^(m_s - m*) ;  out = sum_s w_s O_s / sum_s w_s l_s ;
//   lse = (m* + log2 sum_s w_s l_s) ln 2.
template <int DV>
__global__ __launch_bounds__(DV / 4) void ssa_decode_merge_kernel(const float *__restrict__ part_o,
                                                                   const float *__restrict__ part_ml,
                                                                   uint16_t *__restrict__ out,
                                                                   float *__restrict__ lse, int n_splits)
{
    const int64_t h = blockIdx.x;  // flat (b, query head)
    const float *ml = part_ml + h * n_splits * 2;
    float m_star = LOZA_NEG_INF;
    for (int s = 0; s < n_splits; ++s) m_star = fmaxf(m_star, ml[2 * s]);
    const int c = threadIdx.x * 4;
    if (m_star == LOZA_NEG_INF) {  // no live key at all (empty cache)
        u32x2 z; z[0] = 0; z[1] = 0;
        *(u32x2 *)(out + h * DV + c) = z;
        if (threadIdx.x == 0) lse[h] = LOZA_NEG_INF;
        return;
    }
    float den = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < n_splits; ++s) {
        const float w = __builtin_amdgcn_exp2f(ml[2 * s] - m_star);
        den += w * ml[2 * s + 1];
        const float4 v = *(const float4 *)(part_o + (h * n_splits + s) * DV + c);
        acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
    }
    const float inv = 1.0f / den;
    u32x2 w2;
    w2[0] = pack_bf16(acc.x * inv, acc.y * inv);
    w2[1] = pack_bf16(acc.z * inv, acc.w * inv);
    *(u32x2 *)(out + h * DV + c) = w2;
    if (threadIdx.x == 0) lse[h] = (m_star + __builtin_amdgcn_logf(den)) * 0.69314718055994530942f;
}

// ---------------------------------------------------------------------------------------------------
template <int DQK, int DV, bool ALIAS>
static hipError_t launch_prefill_t(const FwdParams &p, hipStream_t stream)
{
    using C = TileCfg<DQK, DV, 4, 1, ALIAS>;
    auto kern = ssa_fwd_kernel<DQK, DV, 4, 1, ALIAS, false>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int64_t blocks = (int64_t)p.row_tiles * p.Hkv * p.B;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <int DQK, int DV, bool ALIAS>
static hipError_t launch_decode_t(const FwdParams &p, hipStream_t stream)
{
    using C = TileCfg<DQK, DV, 2, 2, ALIAS>;
    auto kern = ssa_fwd_kernel<DQK, DV, 2, 2, ALIAS, true>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int64_t blocks = (int64_t)p.n_splits * p.row_tiles * p.Hkv * p.B;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), C::LDS_BYTES, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ssa_decode_merge_kernel<DV>, dim3((unsigned)((int64_t)p.B * p.Hq)), dim3(DV / 4), 0, stream,
                       p.part_o, p.part_ml, p.out, p.lse, p.n_splits);
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

hipError_t launch_decode_bf16(const FwdParams &p, int d_qk, int d_v, bool alias, hipStream_t stream)
{
    if (d_qk == 576 && d_v == 512 && alias) return launch_decode_t<576, 512, true>(p, stream);
    if (d_qk == 128 && d_v == 128) return alias ? launch_decode_t<128, 128, true>(p, stream)
                                                : launch_decode_t<128, 128, false>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace loza
