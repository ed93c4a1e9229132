// fp32 streaming sparse attention prefill for gfx950: fp32 in, fp32 arithmetic, fp32 out.
//
// O* = softmax(scale * Q K*^T) V* over live(i) = { j <= i : j < n_sink or i - j < window }
// (paper: Architecture section, Eq. 2 / Eq. 4).  This is the small, exact-arithmetic twin of the
// bf16 MFMA kernels: one wavefront owns one query row, walks that row's live keys (sink range,
// then window range, enumerated in closed form) in chunks of 64, one key per lane for the scores
// and one output column per lane for the weighted sum, with an online softmax across chunks.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "ssa_kernels.h"

namespace loza {

constexpr int F32_MAX_D = 256;
constexpr int F32_WAVES = 4;

__global__ __launch_bounds__(64 * F32_WAVES) void ssa_prefill_f32_kernel(const F32Params p)
{
    __shared__ float s_q[F32_WAVES][F32_MAX_D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool decode = p.seqlens != nullptr;
    const int64_t n_rows = decode ? (int64_t)p.B * p.Hq : (int64_t)p.B * p.S * p.Hq;
    const int64_t r = (int64_t)blockIdx.x * F32_WAVES + wave;
    if (r >= n_rows) return;  // whole wavefront leaves together; no block-wide barrier is used
    const int h = (int)(r % p.Hq);
    const int64_t bi = r / p.Hq;
    int i;
    int64_t b;
    if (decode) {
        b = bi;
        const int64_t L = (int64_t)p.seqlens[b] < p.S ? (int64_t)p.seqlens[b] : p.S;  // a length beyond the cache is cut to it
        if (L <= 0) {  // empty cache: out = 0, lse = -inf
            for (int c = lane; c < p.d_v; c += 64) p.out[r * p.d_v + c] = 0.f;
            if (lane == 0) p.lse[r] = -INFINITY;
            return;
        }
        i = (int)(L - 1);
    } else {
        i = (int)(bi % p.S);
        b = bi / p.S;
    }
    const int g = h / (p.Hq / p.Hkv);

    const float *q = p.q + r * p.d_qk;
    for (int c = lane; c < p.d_qk; c += 64) s_q[wave][c] = q[c];
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    // live keys: [0, se) then [wb, i], disjoint and ordered
    const int se = p.n_sink < i + 1 ? p.n_sink : i + 1;
    const int qblk = i / p.block;
    int wb = p.window > qblk ? 0 : (qblk - p.window + 1) * p.block;
    if (wb < se) wb = se;
    const int n_live = se + (i - wb + 1);

    const float *kb = p.k + ((int64_t)b * p.S * p.Hkv + g) * p.k_row;
    const float *vb = p.v + ((int64_t)b * p.S * p.Hkv + g) * p.v_row;
    const int64_t kstep = (int64_t)p.Hkv * p.k_row, vstep = (int64_t)p.Hkv * p.v_row;

    float m = -INFINITY, l = 0.f;
    float acc[F32_MAX_D / 64];
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) acc[c] = 0.f;

    for (int u0 = 0; u0 < n_live; u0 += 64) {
        const int u = u0 + lane;
        const bool have = u < n_live;
        const int j = have ? (u < se ? u : wb + (u - se)) : 0;
        float s = -INFINITY;
        if (have) {
            const float *kr = kb + (int64_t)j * kstep;
            float dot = 0.f;
            for (int c = 0; c < p.d_qk; ++c) dot = fmaf(s_q[wave][c], kr[c], dot);
            s = dot * p.scale;
        }
        float cm = s;
        for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
        const float m_new = fmaxf(m, cm);  // finite: every chunk holds at least one live key
        const float alpha = expf(m - m_new);
        const float pj = have ? expf(s - m_new) : 0.f;
        float ps = pj;
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
        l = l * alpha + ps;
        m = m_new;
#pragma unroll
        for (int c = 0; c < F32_MAX_D / 64; ++c) acc[c] *= alpha;
        const int cnt = n_live - u0 < 64 ? n_live - u0 : 64;
        for (int jj = 0; jj < cnt; ++jj) {
            const float w = __shfl(pj, jj, 64);
            const int jk = __shfl(j, jj, 64);
            const float *vr = vb + (int64_t)jk * vstep;
#pragma unroll
            for (int c = 0; c < F32_MAX_D / 64; ++c) {
                const int col = c * 64 + lane;
                if (col < p.d_v) acc[c] = fmaf(w, vr[col], acc[c]);
            }
        }
    }
    const float inv = 1.0f / l;
    float *o = p.out + r * p.d_v;
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) {
        const int col = c * 64 + lane;
        if (col < p.d_v) o[col] = acc[c] * inv;
    }
    if (lane == 0) p.lse[decode ? r : ((int64_t)b * p.Hq + h) * p.S + i] = m + logf(l);
}

hipError_t launch_prefill_f32(const F32Params &p, hipStream_t stream)
{
    const int64_t n_rows = p.seqlens ? (int64_t)p.B * p.Hq : (int64_t)p.B * p.S * p.Hq;
    const int64_t blocks = (n_rows + F32_WAVES - 1) / F32_WAVES;
    hipLaunchKernelGGL(ssa_prefill_f32_kernel, dim3((unsigned)blocks), dim3(64 * F32_WAVES), 0, stream, p);
    return hipGetLastError();
}

// ---- fp32 backward (the small, exact-arithmetic twin of ssa_bwd.hip) --------------------------------
// With p_ij = exp(scale q_i.k_j - lse_i) over live pairs, D_i = dO_i . O_i, dP_ij = dO_i . v_j and
// dS_ij = p_ij (dP_ij - D_i):   dQ_i = scale sum_j dS_ij k_j,  dK_j = scale sum_i dS_ij q_i,
// dV_j = sum_i p_ij dO_i   (the derivative of the paper's Eq. 4; Architecture section, Training).
// Two kernels, no atomics: one wavefront per query row walks that row's live keys (dQ); one wavefront
// per key walks the query rows that see it (dK, dV), 64 at a time, one per lane for the scalars and
// one gradient column per lane for the sums.

// per-lane dot product of two rows of n floats
static __device__ __forceinline__ float dot_rows(const float *a, const float *b, int n)
{
    float d = 0.f;
    for (int c = 0; c < n; ++c) d = fmaf(a[c], b[c], d);
    return d;
}

__global__ __launch_bounds__(64 * F32_WAVES) void ssa_backward_f32_dq_kernel(const F32BwdParams p)
{
    __shared__ float s_q[F32_WAVES][F32_MAX_D], s_do[F32_WAVES][F32_MAX_D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq;
    const int64_t r = (int64_t)blockIdx.x * F32_WAVES + wave;
    if (r >= n_rows) return;  // whole wavefront leaves together; no block-wide barrier is used
    const int h = (int)(r % p.Hq);
    const int64_t bi = r / p.Hq;
    const int i = (int)(bi % p.S);
    const int64_t b = bi / p.S;
    const int g = h / (p.Hq / p.Hkv);

    float dpart = 0.f;  // D = dO . O
    for (int c = lane; c < p.d_qk; c += 64) s_q[wave][c] = p.q[r * p.d_qk + c];
    for (int c = lane; c < p.d_v; c += 64) {
        const float d = p.dout[r * p.d_v + c];
        s_do[wave][c] = d;
        dpart = fmaf(d, p.out[r * p.d_v + c], dpart);
    }
    for (int off = 32; off > 0; off >>= 1) dpart += __shfl_xor(dpart, off, 64);
    const float D = dpart;
    const float lse = p.lse[((int64_t)b * p.Hq + h) * p.S + i];
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    const int se = p.n_sink < i + 1 ? p.n_sink : i + 1;
    const int qblk = i / p.block;
    int wb = p.window > qblk ? 0 : (qblk - p.window + 1) * p.block;
    if (wb < se) wb = se;
    const int n_live = se + (i - wb + 1);
    const float *kb = p.k + ((int64_t)b * p.S * p.Hkv + g) * p.k_row;
    const float *vb = p.v + ((int64_t)b * p.S * p.Hkv + g) * p.v_row;
    const int64_t kstep = (int64_t)p.Hkv * p.k_row, vstep = (int64_t)p.Hkv * p.v_row;

    float acc[F32_MAX_D / 64];
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) acc[c] = 0.f;
    for (int u0 = 0; u0 < n_live; u0 += 64) {
        const int u = u0 + lane;
        const bool have = u < n_live;
        const int j = have ? (u < se ? u : wb + (u - se)) : 0;
        float ds = 0.f;
        if (have) {
            const float s = dot_rows(s_q[wave], kb + (int64_t)j * kstep, p.d_qk) * p.scale;
            const float pj = expf(s - lse);
            const float dp = dot_rows(s_do[wave], vb + (int64_t)j * vstep, p.d_v);
            ds = pj * (dp - D);
        }
        const int cnt = n_live - u0 < 64 ? n_live - u0 : 64;
        for (int jj = 0; jj < cnt; ++jj) {
            const float w = __shfl(ds, jj, 64);
            const float *kr = kb + (int64_t)__shfl(j, jj, 64) * kstep;
#pragma unroll
            for (int c = 0; c < F32_MAX_D / 64; ++c) {
                const int col = c * 64 + lane;
                if (col < p.d_qk) acc[c] = fmaf(w, kr[col], acc[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) {
        const int col = c * 64 + lane;
        if (col < p.d_qk) p.dq[r * p.d_qk + col] = acc[c] * p.scale;
    }
}

__global__ __launch_bounds__(64 * F32_WAVES) void ssa_backward_f32_dkv_kernel(const F32BwdParams p)
{
    __shared__ float s_k[F32_WAVES][F32_MAX_D], s_v[F32_WAVES][F32_MAX_D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t n_keys = (int64_t)p.B * p.S * p.Hkv;
    const int64_t kr_idx = (int64_t)blockIdx.x * F32_WAVES + wave;  // flat (b, j, g)
    if (kr_idx >= n_keys) return;
    const int g = (int)(kr_idx % p.Hkv);
    const int64_t bj = kr_idx / p.Hkv;
    const int j = (int)(bj % p.S);
    const int64_t b = bj / p.S;
    const int G = p.Hq / p.Hkv;

    for (int c = lane; c < p.d_qk; c += 64) s_k[wave][c] = p.k[kr_idx * p.k_row + c];
    for (int c = lane; c < p.d_v; c += 64) s_v[wave][c] = p.v[kr_idx * p.v_row + c];
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    // the positions that see key j: every later one for a sink key, else those whose window still
    // holds it: i / block - window + 1 <= j / block
    int64_t i_last = p.S - 1;
    if (j >= p.n_sink) {
        const int64_t jb = j / p.block, last_blk = (p.S - 1) / p.block;
        if (jb + p.window - 1 < last_blk) i_last = (jb + p.window) * p.block - 1;  // (< S: no overflow)
    }
    const int64_t n_rows = (i_last - j + 1) * G;  // rows (i, head of the group), position-major

    float acc_k[F32_MAX_D / 64], acc_v[F32_MAX_D / 64];
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) { acc_k[c] = 0.f; acc_v[c] = 0.f; }
    for (int64_t u0 = 0; u0 < n_rows; u0 += 64) {
        const int64_t u = u0 + lane;
        const bool have = u < n_rows;
        float pj = 0.f, ds = 0.f;
        if (have) {
            const int64_t i = j + u / G;
            const int h = g * G + (int)(u % G);
            const int64_t row = ((int64_t)b * p.S + i) * p.Hq + h;  // flat (b, i, h)
            const float *qr = p.q + row * p.d_qk, *dor = p.dout + row * p.d_v;
            const float s = dot_rows(qr, s_k[wave], p.d_qk) * p.scale;
            pj = expf(s - p.lse[((int64_t)b * p.Hq + h) * p.S + i]);
            const float dp = dot_rows(dor, s_v[wave], p.d_v);
            const float D = dot_rows(dor, p.out + row * p.d_v, p.d_v);
            ds = pj * (dp - D);
        }
        const int cnt = n_rows - u0 < 64 ? (int)(n_rows - u0) : 64;
        for (int jj = 0; jj < cnt; ++jj) {
            const float wk = __shfl(ds, jj, 64), wv = __shfl(pj, jj, 64);
            const int64_t uu = u0 + jj;
            const int64_t rr = ((int64_t)b * p.S + j + uu / G) * p.Hq + g * G + (int)(uu % G);
            const float *qr = p.q + rr * p.d_qk, *dor = p.dout + rr * p.d_v;
#pragma unroll
            for (int c = 0; c < F32_MAX_D / 64; ++c) {
                const int col = c * 64 + lane;
                if (col < p.d_qk) acc_k[c] = fmaf(wk, qr[col], acc_k[c]);
                if (col < p.d_v) acc_v[c] = fmaf(wv, dor[col], acc_v[c]);
            }
        }
    }
    // values that are a prefix of the key rows: one tensor, one gradient (dK with dV added to its
    // first d_v columns), and no dv is written
#pragma unroll
    for (int c = 0; c < F32_MAX_D / 64; ++c) {
        const int col = c * 64 + lane;
        if (p.dv == nullptr) {
            if (col < p.d_qk) p.dk[kr_idx * p.d_qk + col] = acc_k[c] * p.scale + (col < p.d_v ? acc_v[c] : 0.f);
        } else {
            if (col < p.d_qk) p.dk[kr_idx * p.d_qk + col] = acc_k[c] * p.scale;
            if (col < p.d_v) p.dv[kr_idx * p.d_v + col] = acc_v[c];
        }
    }
}

hipError_t launch_backward_f32(const F32BwdParams &p, hipStream_t stream)
{
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq, n_keys = (int64_t)p.B * p.S * p.Hkv;
    hipLaunchKernelGGL(ssa_backward_f32_dq_kernel, dim3((unsigned)((n_rows + F32_WAVES - 1) / F32_WAVES)), dim3(64 * F32_WAVES), 0,
                       stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ssa_backward_f32_dkv_kernel, dim3((unsigned)((n_keys + F32_WAVES - 1) / F32_WAVES)), dim3(64 * F32_WAVES), 0,
                       stream, p);
    return hipGetLastError();
}

}  // namespace loza
