// Shared device-side helpers for the gfx950 kernels (wave = 64 lanes).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sp_types.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

#define SP_WAVE 64

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// fp32 -> bf16, round to nearest even (the hardware conversion on gfx950).
__device__ __forceinline__ bf16_t f2bf(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(bf16_t, b);
}

__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
    return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// erf by the five-term rational approximation of Abramowitz & Stegun 7.1.26 (absolute
// error < 1.5e-7, far below the bf16 rounding of what it feeds): branch-free, one exp and
// one reciprocal.  Returns erf(|x| / sqrt 2) and exp(-x^2 / 2).
__device__ __forceinline__ float erf_abs_half(float x, float* gauss) {
    const float z = fabsf(x) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * z);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    *gauss = __expf(-z * z);
    return 1.0f - poly * *gauss;
}
// Exact-erf GELU x Phi(x), Phi the standard normal distribution function, written as
// max(x, 0) - |x| Phi(-|x|): no cancellation in the negative tail.  log2 Phi(-a) is close to a
// parabola; a degree-6 minimax polynomial on [0, 6] is within 6.5e-5 of it (Phi(-a) to 4.5e-5
// relative, the result to 7e-6 absolute and 3 % of a bf16 rounding step), beyond 6 the term is
// below 6e-9 and a is clamped.  9 VALU operations and one v_exp_f32 per value: in a GEMM epilogue
// the function is VALU-bound (the erf form above costs 14 + exp + rcp).
__device__ __forceinline__ float gelu_erf(float x) {
    const float a = fminf(fabsf(x), 6.0f);
    float p = 2.299006353e-05f;
    p = fmaf(p, a, -6.111000662e-04f);
    p = fmaf(p, a, 7.195565668e-03f);
    p = fmaf(p, a, -5.118533638e-02f);
    p = fmaf(p, a, -4.612719268e-01f);
    p = fmaf(p, a, -1.150174254e+00f);
    p = fmaf(p, a, -1.000064790e+00f);
    return fmaf(-fabsf(x), __builtin_amdgcn_exp2f(p), fmaxf(x, 0.0f));
}
// Its derivative: 0.5 (1 + erf(x / sqrt 2)) + x exp(-x^2 / 2) / sqrt(2 pi).
__device__ __forceinline__ float gelu_erf_grad(float x) {
    float gs;
    const float e = erf_abs_half(x, &gs);
    return 0.5f * (1.0f + copysignf(e, x)) + x * gs * 0.39894228040143267794f;
}

// Sum / max over the 64 lanes of a wave; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a 256-thread block (4 waves); `red` is 4 floats of LDS per call site.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// Work-group order that keeps neighbouring tiles on one XCD: hardware deals
// consecutive work-group ids round-robin over the 8 XCDs (each with its own
// L2), so id i is remapped to the i-th slot of "its" XCD's contiguous range.
__device__ __forceinline__ int xcd_remap(int pid, int nblocks) {
    const int xcd = pid & 7, q = pid >> 3;
    const int per = nblocks >> 3, rem = nblocks & 7;
    return xcd * per + (xcd < rem ? xcd : rem) + q;
}

// Second stage of the deterministic column reductions: out[c] = sum over partial rows p of
// part[p * ld + c].  A work-group covers 64 columns; its four waves each add every fourth
// row with four independent accumulators (loads in flight instead of one dependent chain),
// then the 16 partial sums of a column are added in a fixed order.
__device__ __forceinline__ void colsum_rows_body(const float* __restrict__ part, int nparts, int ld, int n,
                                                 float* __restrict__ out, float* lds /* [4][64] */) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (c < n) {
        int p = w;
        for (; p + 12 < nparts; p += 16) {
            a0 += part[(size_t)p * ld + c];
            a1 += part[(size_t)(p + 4) * ld + c];
            a2 += part[(size_t)(p + 8) * ld + c];
            a3 += part[(size_t)(p + 12) * ld + c];
        }
        for (; p < nparts; p += 4) a0 += part[(size_t)p * ld + c];
    }
    lds[w * 64 + lane] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (w == 0 && c < n) out[c] = (lds[lane] + lds[64 + lane]) + (lds[128 + lane] + lds[192 + lane]);
}
