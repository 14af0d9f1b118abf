// Row normalisation feeding the bf16 GEMMs: RMSNorm (decoder) and LayerNorm
// (encoder).  HBM-bound.  Launches of many rows: one WAVE per token row (four rows
// per 256-thread work-group), so the reductions are wave shuffles only -- no LDS,
// no barrier.  Launches of few rows: one work-group per row (second kernel below).
// A lane issues all of its 16-byte loads of the row at once (VPL of them, the
// row stays in registers), and the row is written once as bf16.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int NORM_THREADS = 256;
constexpr int NORM_ROWS = NORM_THREADS / SP_WAVE;   // rows per work-group

// VPL = float4 per lane: d <= 256 * VPL.
template <bool LAYERNORM, int VPL>
__global__ __launch_bounds__(NORM_THREADS) void norm_kernel(const float* __restrict__ h,
                                                            const bf16_t* __restrict__ gain,
                                                            const bf16_t* __restrict__ bias,
                                                            bf16_t* __restrict__ out, int T, int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * NORM_ROWS + (threadIdx.x >> 6);
    if (row >= T) return;                       // whole waves leave; nothing below synchronises
    const float4* src = reinterpret_cast<const float4*>(h + (size_t)row * d);
    const int nv = d >> 2;
    float4 v[VPL];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int idx = lane + i * SP_WAVE;
        if (idx < nv) v[i] = src[idx];
    }
    // Gain and bias of the lane's columns: fetched here, behind the row's loads and ahead of the
    // reductions, when the registers allow; fetched where they are used, each little load is
    // waited for in turn (eight cache round trips at the end of a 1280-wide row).
    constexpr bool PRE = VPL <= 8;
    const uint2* g2 = reinterpret_cast<const uint2*>(gain);
    const uint2* b2 = reinterpret_cast<const uint2*>(bias);
    uint2 gv[PRE ? VPL : 1], bv[PRE ? VPL : 1];
    if (PRE) {
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int idx = lane + i * SP_WAVE;
            if (idx < nv) {
                gv[i] = g2[idx];
                if (LAYERNORM) bv[i] = b2[idx];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int idx = lane + i * SP_WAVE;
        if (idx < nv)
            s += LAYERNORM ? (v[i].x + v[i].y) + (v[i].z + v[i].w)
                           : (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    }
    float mean = 0.f, r;
    if (LAYERNORM) {
        mean = wave_sum(s) / (float)d;
        float c = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int idx = lane + i * SP_WAVE;
            if (idx < nv) {
                const float a = v[i].x - mean, b = v[i].y - mean, e = v[i].z - mean, f = v[i].w - mean;
                c += (a * a + b * b) + (e * e + f * f);
            }
        }
        r = rsqrtf(wave_sum(c) / (float)d + eps);
    } else {
        r = rsqrtf(wave_sum(s) / (float)d + eps);
    }
    uint2* dst = reinterpret_cast<uint2*>(out + (size_t)row * d);
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int idx = lane + i * SP_WAVE;
        if (idx < nv) {
            const uint2 g = PRE ? gv[PRE ? i : 0] : g2[idx];
            float o0 = (v[i].x - mean) * r * bf_lo(g.x), o1 = (v[i].y - mean) * r * bf_hi(g.x);
            float o2 = (v[i].z - mean) * r * bf_lo(g.y), o3 = (v[i].w - mean) * r * bf_hi(g.y);
            if (LAYERNORM) {
                const uint2 b = PRE ? bv[PRE ? i : 0] : b2[idx];
                o0 += bf_lo(b.x); o1 += bf_hi(b.x); o2 += bf_lo(b.y); o3 += bf_hi(b.y);
            }
            dst[idx] = make_uint2(pack_bf2(o0, o1), pack_bf2(o2, o3));
        }
    }
}

// One 256-thread work-group per row (reductions through 4 floats of LDS): four times the waves
// of the kernel above, which is what a launch of few rows needs to keep enough loads in flight.
constexpr int NORM_BLOCK_MAXV = 8;  // float4 per thread -> d <= 8192

template <bool LAYERNORM>
__global__ __launch_bounds__(NORM_THREADS) void norm_block_kernel(const float* __restrict__ h,
                                                            const bf16_t* __restrict__ gain,
                                                            const bf16_t* __restrict__ bias,
                                                            bf16_t* __restrict__ out, int d, float eps) {
    __shared__ float red[8];
    const int row = blockIdx.x;
    const float4* src = reinterpret_cast<const float4*>(h + (size_t)row * d);
    const int nv = d >> 2;
    float4 v[NORM_BLOCK_MAXV];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_BLOCK_MAXV; ++i) {
        const int idx = threadIdx.x + i * NORM_THREADS;
        if (idx < nv) {
            v[i] = src[idx];
            s += LAYERNORM ? (v[i].x + v[i].y) + (v[i].z + v[i].w)
                           : (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
        }
    }
    // gain and bias of the thread's columns, fetched ahead of the reductions (see norm_kernel)
    const uint2* g2 = reinterpret_cast<const uint2*>(gain);
    const uint2* b2 = reinterpret_cast<const uint2*>(bias);
    uint2 gv[NORM_BLOCK_MAXV], bv[NORM_BLOCK_MAXV];
#pragma unroll
    for (int i = 0; i < NORM_BLOCK_MAXV; ++i) {
        const int idx = threadIdx.x + i * NORM_THREADS;
        if (idx < nv) {
            gv[i] = g2[idx];
            if (LAYERNORM) bv[i] = b2[idx];
        }
    }
    float mean = 0.f, r;
    if (LAYERNORM) {
        mean = block_sum_256(s, red) / (float)d;
        float c = 0.f;
#pragma unroll
        for (int i = 0; i < NORM_BLOCK_MAXV; ++i) {
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
#pragma unroll
    for (int i = 0; i < NORM_BLOCK_MAXV; ++i) {
        const int idx = threadIdx.x + i * NORM_THREADS;
        if (idx < nv) {
            const uint2 g = gv[i];
            float o0 = (v[i].x - mean) * r * bf_lo(g.x), o1 = (v[i].y - mean) * r * bf_hi(g.x);
            float o2 = (v[i].z - mean) * r * bf_lo(g.y), o3 = (v[i].w - mean) * r * bf_hi(g.y);
            if (LAYERNORM) {
                const uint2 b = bv[i];
                o0 += bf_lo(b.x); o1 += bf_hi(b.x); o2 += bf_lo(b.y); o3 += bf_hi(b.y);
            }
            dst[idx] = make_uint2(pack_bf2(o0, o1), pack_bf2(o2, o3));
        }
    }
}

template <bool LN>
void launch_norm(hipStream_t st, const float* h, const bf16_t* gain, const bf16_t* bias, bf16_t* out, int T, int d,
                 float eps) {
    // fewer than ~32 row-waves per CU: spread each row over a whole work-group instead
    if (T < 8192) {
        norm_block_kernel<LN><<<T, NORM_THREADS, 0, st>>>(h, gain, bias, out, d, eps);
        return;
    }
    const int grid = (T + NORM_ROWS - 1) / NORM_ROWS;
    if (d <= 256 * 8)
        norm_kernel<LN, 8><<<grid, NORM_THREADS, 0, st>>>(h, gain, bias, out, T, d, eps);
    else if (d <= 256 * 16)
        norm_kernel<LN, 16><<<grid, NORM_THREADS, 0, st>>>(h, gain, bias, out, T, d, eps);
    else
        norm_kernel<LN, 32><<<grid, NORM_THREADS, 0, st>>>(h, gain, bias, out, T, d, eps);
}

}  // namespace

hipError_t spk_launch_norm(hipStream_t st, const float* h, const bf16_t* gain, const bf16_t* bias,
                           bf16_t* out, int T, int d, float eps) {
    if (T <= 0) return hipSuccess;
    if (d <= 0 || (d & 3) || d > 256 * 32) return hipErrorInvalidValue;
    if (bias)
        launch_norm<true>(st, h, gain, bias, out, T, d, eps);
    else
        launch_norm<false>(st, h, gain, nullptr, out, T, d, eps);
    return hipGetLastError();
}
