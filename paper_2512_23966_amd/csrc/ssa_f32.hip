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
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq;
    const int64_t r = (int64_t)blockIdx.x * F32_WAVES + wave;
    if (r >= n_rows) return;  // whole wavefront leaves together; no block-wide barrier is used
    const int h = (int)(r % p.Hq);
    const int64_t bi = r / p.Hq;
    const int i = (int)(bi % p.S);
    const int64_t b = bi / p.S;
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
    if (lane == 0) p.lse[((int64_t)b * p.Hq + h) * p.S + i] = m + logf(l);
}

hipError_t launch_prefill_f32(const F32Params &p, hipStream_t stream)
{
    const int64_t n_rows = (int64_t)p.B * p.S * p.Hq;
    const int64_t blocks = (n_rows + F32_WAVES - 1) / F32_WAVES;
    hipLaunchKernelGGL(ssa_prefill_f32_kernel, dim3((unsigned)blocks), dim3(64 * F32_WAVES), 0, stream, p);
    return hipGetLastError();
}

}  // namespace loza
