// Device-side helpers shared by the kernel translation units.
#ifndef LOZA_SSA_DEVICE_H
#define LOZA_SSA_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace loza {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef __attribute__((address_space(1))) const void *glb_void_ptr;

#define LOZA_NEG_INF (-__builtin_inff())

// Scalar (wave-uniform) load of one dword through a buffer resource: the LLVM intrinsic behind
// s_buffer_load_dword. The compiler tracks it like any other load (it waits before the first use).
__device__ int32_t llvm_amdgcn_s_buffer_load_i32(i32x4 rsrc, int32_t byte_offset, int32_t cachepolicy) __asm("llvm.amdgcn.s.buffer.load.i32");

// Buffer resource (gfx9 layout) over `entries` consecutive int32 values at `base`: raw buffer, no
// stride, the size in bytes as its range (reads beyond it return 0), 32-bit data format.
static __device__ __forceinline__ i32x4 table_row_resource(const int32_t *base, int entries)
{
    const uint64_t a = (uint64_t)base;
    i32x4 r;
    r[0] = (int32_t)(uint32_t)a;
    r[1] = (int32_t)((uint32_t)(a >> 32) & 0xffffu);
    r[2] = entries * 4;
    r[3] = 0x00020000;
    return r;
}

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

// max(x, value of x in the lane of the other wavefront half (lane ^ 32)), without touching LDS.
static __device__ __forceinline__ float max_with_other_half(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    // v_permlane32_swap exchanges one half of its first operand with the opposite half of the
    // second; fed with two copies of x, one result holds the low half's values in both halves and
    // the other the high half's, so their maximum is the wanted value in every lane
    // (the copy and both results go through empty asm statements: the optimiser otherwise folds
    // the maximum of the two results of a swap into the first result alone)
    uint32_t u2 = u;
    asm volatile("" : "+v"(u2));
    const auto r = __builtin_amdgcn_permlane32_swap(u, u2, false, false);
    uint32_t r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    return fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}

static __device__ __forceinline__ float xor32(float x)
{
    // value held by the lane in the other half of the wavefront (lane ^ 32)
    return __shfl_xor(x, 32, 64);
}

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (gfx9 encoding:
// vmcnt[3:0] in bits 3:0 and vmcnt[5:4] in bits 15:14; expcnt and lgkmcnt fields left at "no wait")
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// First key of the window of query i: the window holds the `window` most recent blocks of `block`
// tokens, the query's own block included (block = 1: the `window` most recent tokens).
__device__ __forceinline__ int window_begin_of(int i, int window, int block)
{
    const int qb = block == 1 ? i : i / block;
    return window > qb ? 0 : (qb - window + 1) * block;
}

// Prefill tiles that start below this position are computed with two-term P (p = hi + lo, both
// bf16) from the outset: with so few live keys the output is as large as single value rows, and the
// bf16 rounding of P would be a visible share of the error budget there.
constexpr int kPrecisePositions = 128;

// Everywhere else the weights are rounded to bf16 once (relative error 2^-9 each), which reaches the
// output as at most 2^-9 times the weighted mean distance of the value rows from the output. That is
// harmless next to the output's own rounding while |out| < 2 (half an ulp of bf16 is at most 2^-8 there,
// of a budget of 1e-2); from 2 on the rounding of the result alone takes 2^-7. Such results only come
// from rows whose weight sits on a handful of keys, which is also where the rounding of P shows most:
// a prefill tile that produced one (|out| >= this, a little below 2 so that the test cannot miss a
// result just above it) is computed again with two-term P, and a decode query that did is computed
// again by the merge kernel, directly in fp32.
constexpr float kRedoMagnitude = 1.96875f;

// A decode query with fewer live keys than this is not worth a matrix-core pass and, with so few
// terms, would show the bf16 rounding of the softmax weights in its output: the split kernel leaves
// it alone and the merge kernel computes it directly in fp32.
constexpr int kDirectKeys = 128;

}  // namespace loza
#endif
