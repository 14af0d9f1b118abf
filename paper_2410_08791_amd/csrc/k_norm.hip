// Row normalisation feeding the bf16 GEMMs: RMSNorm (decoder) and LayerNorm
// (encoder).  HBM-bound: one 256-thread work-group per token row, the row is
// read once with 16-byte loads, kept in registers, reduced with wave shuffles
// plus 4 floats of LDS, and written once as bf16.
#include "sp_kernels.h"

namespace {

constexpr int NORM_THREADS = 256;
constexpr int NORM_MAXV = 8;  // float4 per thread -> d <= 8192

template <bool LAYERNORM>
__global__ __launch_bounds__(NORM_THREADS) void norm_kernel(const float* __restrict__ h,
                                                            const bf16_t* __restrict__ gain,
                                                            const bf16_t* __restrict__ bias,
                                                            bf16_t* __restrict__ out, int d, float eps) {
    __shared__ float red[8];
    const int row = blockIdx.x;
    const float4* src = reinterpret_cast<const float4*>(h + (size_t)row * d);
    const int nv = d >> 2;
    float4 v[NORM_MAXV];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAXV; ++i) {
        const int idx = threadIdx.x + i * NORM_THREADS;
        if (idx < nv) {
            v[i] = src[idx];
            s += LAYERNORM ? (v[i].x + v[i].y) + (v[i].z + v[i].w)
                           : (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
        }
    }
    float mean = 0.f, r;
    if (LAYERNORM) {
        mean = block_sum_256(s, red) / (float)d;
        float c = 0.f;
#pragma unroll
        for (int i = 0; i < NORM_MAXV; ++i) {
            const int idx = threadIdx.x + i * NORM_THREADS;
            if (idx < nv) {
                const float a = v[i].x - mean, b = v[i].y - mean, e = v[i].z - mean, f = v[i].w - mean;
                c += (a * a + b * b) + (e * e + f * f);
            }
        }
        r = rsqrtf(block_sum_256(c, red + 4) / (float)d + eps);
    } else {
        r = rsqrtf(block_sum_256(s, red) / (float)d + eps);
    }
    uint2* dst = reinterpret_cast<uint2*>(out + (size_t)row * d);
    const uint2* g2 = reinterpret_cast<const uint2*>(gain);
    const uint2* b2 = reinterpret_cast<const uint2*>(bias);
#pragma unroll
    for (int i = 0; i < NORM_MAXV; ++i) {
        const int idx = threadIdx.x + i * NORM_THREADS;
        if (idx < nv) {
            const uint2 g = g2[idx];
            float o0 = (v[i].x - mean) * r * bf_lo(g.x), o1 = (v[i].y - mean) * r * bf_hi(g.x);
            float o2 = (v[i].z - mean) * r * bf_lo(g.y), o3 = (v[i].w - mean) * r * bf_hi(g.y);
            if (LAYERNORM) {
                const uint2 b = b2[idx];
                o0 += bf_lo(b.x); o1 += bf_hi(b.x); o2 += bf_lo(b.y); o3 += bf_hi(b.y);
            }
            dst[idx] = make_uint2(pack_bf2(o0, o1), pack_bf2(o2, o3));
        }
    }
}

}  // namespace

hipError_t spk_launch_norm(hipStream_t st, const float* h, const bf16_t* gain, const bf16_t* bias,
                           bf16_t* out, int T, int d, float eps) {
    if (T <= 0) return hipSuccess;
    if (d <= 0 || (d & 3) || d > NORM_THREADS * NORM_MAXV * 4) return hipErrorInvalidValue;
    if (bias)
        norm_kernel<true><<<T, NORM_THREADS, 0, st>>>(h, gain, bias, out, d, eps);
    else
        norm_kernel<false><<<T, NORM_THREADS, 0, st>>>(h, gain, nullptr, out, d, eps);
    return hipGetLastError();
}
