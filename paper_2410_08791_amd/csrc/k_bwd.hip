// HBM-bound kernels of the backward pass: MSE loss and its gradient, SwiGLU
// backward, RMSNorm backward (with the deterministic two-stage reduction of
// the gain gradient), fp32 -> bf16 copies, rowsum(dO * O).  No atomics: every
// reduction has a fixed order, so gradients are bit-identical from run to run
// and across window settings.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int TH = 256;

// ---- loss = mean((y - t)^2), dy = 2 (y - t) / n -----------------------------------
__global__ __launch_bounds__(TH) void mse_partial_kernel(const float* __restrict__ y, const float* __restrict__ t,
                                                         float* __restrict__ dy, bf16_t* __restrict__ dyb,
                                                         float* __restrict__ part, size_t n, float two_over_n) {
    __shared__ float red[4];
    float s = 0.f;
    for (size_t i = (size_t)blockIdx.x * TH + threadIdx.x; i < n; i += (size_t)gridDim.x * TH) {
        const float d = y[i] - t[i];
        s += d * d;
        const float g = d * two_over_n;
        dy[i] = g;
        dyb[i] = f2bf(g);
    }
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) part[blockIdx.x] = s;
}

__global__ __launch_bounds__(TH) void mse_final_kernel(const float* __restrict__ part, int nparts,
                                                       float* __restrict__ loss, float inv_n) {
    __shared__ float red[4];
    float s = 0.f;
    for (int i = threadIdx.x; i < nparts; i += TH) s += part[i];
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) *loss = s * inv_n;
}

// ---- SwiGLU backward, in place over gu = [g | u] -------------------------------------
__global__ __launch_bounds__(TH) void swiglu_bwd_kernel(const bf16_t* __restrict__ dz, bf16_t* __restrict__ gu,
                                                        int T, int f) {
    const int fc = f >> 3;
    const size_t total = (size_t)T * fc;
    for (size_t i = (size_t)blockIdx.x * TH + threadIdx.x; i < total; i += (size_t)gridDim.x * TH) {
        const size_t t = i / fc;
        const int c = (int)(i - t * fc);
        bf16_t* gp = gu + t * 2 * (size_t)f + c * 8;
        bf16_t* up = gp + f;
        const u32x4_t g = *reinterpret_cast<const u32x4_t*>(gp);
        const u32x4_t u = *reinterpret_cast<const u32x4_t*>(up);
        const u32x4_t d = *reinterpret_cast<const u32x4_t*>(dz + t * (size_t)f + c * 8);
        u32x4_t dg, du;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float o[4];
#pragma unroll
            for (int hsel = 0; hsel < 2; ++hsel) {
                const float gv = hsel ? bf_hi(g[k]) : bf_lo(g[k]);
                const float uv = hsel ? bf_hi(u[k]) : bf_lo(u[k]);
                const float dv = hsel ? bf_hi(d[k]) : bf_lo(d[k]);
                const float sg = 1.0f / (1.0f + __expf(-gv));
                o[hsel] = dv * uv * (sg * (1.0f + gv * (1.0f - sg)));   // d/dg
                o[2 + hsel] = dv * (gv * sg);                           // d/du
            }
            dg[k] = pack_bf2(o[0], o[1]);
            du[k] = pack_bf2(o[2], o[3]);
        }
        *reinterpret_cast<u32x4_t*>(gp) = dg;
        *reinterpret_cast<u32x4_t*>(up) = du;
    }
}

// ---- RMSNorm backward -----------------------------------------------------------------
// a = h r g, r = rsqrt(mean(h^2)+eps).  Given da:  dh_io += r (da g) - h r^3 mean(da g h);
// dgain = sum_t da h r.  Block b owns rows b, b+G, ...; each thread keeps the gain
// gradient of its columns in registers and writes one partial row per block.
constexpr int NB_MAXV = 8;   // float4 per thread -> d <= 8192

__global__ __launch_bounds__(TH) void rmsnorm_bwd_kernel(const float* __restrict__ da, const float* __restrict__ h,
                                                         const bf16_t* __restrict__ gain, float* __restrict__ dh_io,
                                                         bf16_t* __restrict__ dhb, float* __restrict__ part, int T,
                                                         int d, float eps) {
    __shared__ float red[8];
    const int nv = d >> 2;
    float4 gacc[NB_MAXV], gv[NB_MAXV];
#pragma unroll
    for (int i = 0; i < NB_MAXV; ++i) {
        gacc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        const int idx = threadIdx.x + i * TH;
        if (idx < nv) {
            const uint2 g = reinterpret_cast<const uint2*>(gain)[idx];
            gv[i] = make_float4(bf_lo(g.x), bf_hi(g.x), bf_lo(g.y), bf_hi(g.y));
        }
    }
    for (int row = blockIdx.x; row < T; row += gridDim.x) {
        const float4* hp = reinterpret_cast<const float4*>(h + (size_t)row * d);
        const float4* ap = reinterpret_cast<const float4*>(da + (size_t)row * d);
        float4 hv[NB_MAXV], av[NB_MAXV];
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int i = 0; i < NB_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                hv[i] = hp[idx];
                av[i] = ap[idx];
                ss += (hv[i].x * hv[i].x + hv[i].y * hv[i].y) + (hv[i].z * hv[i].z + hv[i].w * hv[i].w);
                dot += (av[i].x * gv[i].x * hv[i].x + av[i].y * gv[i].y * hv[i].y) +
                       (av[i].z * gv[i].z * hv[i].z + av[i].w * gv[i].w * hv[i].w);
            }
        }
        ss = block_sum_256(ss, red);
        dot = block_sum_256(dot, red + 4);
        const float r = rsqrtf(ss / (float)d + eps);
        const float c = r * r * r * dot / (float)d;
        float4* op = reinterpret_cast<float4*>(dh_io + (size_t)row * d);
        uint2* bp = reinterpret_cast<uint2*>(dhb + (size_t)row * d);
#pragma unroll
        for (int i = 0; i < NB_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                float4 o = op[idx];
                o.x += r * av[i].x * gv[i].x - hv[i].x * c;
                o.y += r * av[i].y * gv[i].y - hv[i].y * c;
                o.z += r * av[i].z * gv[i].z - hv[i].z * c;
                o.w += r * av[i].w * gv[i].w - hv[i].w * c;
                op[idx] = o;
                bp[idx] = make_uint2(pack_bf2(o.x, o.y), pack_bf2(o.z, o.w));
                gacc[i].x += av[i].x * hv[i].x * r;
                gacc[i].y += av[i].y * hv[i].y * r;
                gacc[i].z += av[i].z * hv[i].z * r;
                gacc[i].w += av[i].w * hv[i].w * r;
            }
        }
    }
    float4* pp = reinterpret_cast<float4*>(part + (size_t)blockIdx.x * d);
#pragma unroll
    for (int i = 0; i < NB_MAXV; ++i) {
        const int idx = threadIdx.x + i * TH;
        if (idx < nv) pp[idx] = gacc[i];
    }
}


// The same for rows of at most 2048 elements with ONE WAVE PER ROW: a lane holds d/64 elements of
// the row (at most eight float4), the two row sums are wave shuffles, and no barrier separates
// the rows, so a work-group of eight waves keeps eight rows' loads in flight (the
// row-per-work-group form above spends most of its time in its four barriers per row: 2.4 TB/s on
// 8192 x 2048).  The waves' gain-gradient partials are added into LDS in wave order at the end:
// one partial row per work-group.
constexpr int NW_MAXV = 8;    // float4 per lane -> d <= 2048
constexpr int NW_WAVES = 8;

__global__ __launch_bounds__(NW_WAVES * 64) void rmsnorm_bwd_wave_kernel(
    const float* __restrict__ da, const float* __restrict__ h, const bf16_t* __restrict__ gain, float* __restrict__ dh_io,
    bf16_t* __restrict__ dhb, float* __restrict__ part, int T, int d, float eps) {
    __shared__ float4 lds[64 * NW_MAXV];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nv = d >> 2;
    float4 gacc[NW_MAXV], gv[NW_MAXV];
#pragma unroll
    for (int i = 0; i < NW_MAXV; ++i) {
        gacc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        const int idx = lane + i * 64;
        if (idx < nv) {
            const uint2 g = reinterpret_cast<const uint2*>(gain)[idx];
            gv[i] = make_float4(bf_lo(g.x), bf_hi(g.x), bf_lo(g.y), bf_hi(g.y));
        }
    }
    for (int row = blockIdx.x * NW_WAVES + wave; row < T; row += gridDim.x * NW_WAVES) {
        const float4* hp = reinterpret_cast<const float4*>(h + (size_t)row * d);
        const float4* ap = reinterpret_cast<const float4*>(da + (size_t)row * d);
        float4* op = reinterpret_cast<float4*>(dh_io + (size_t)row * d);
        float4 hv[NW_MAXV], av[NW_MAXV], ov[NW_MAXV];
#pragma unroll
        for (int i = 0; i < NW_MAXV; ++i) {
            const int idx = lane + i * 64;
            if (idx < nv) { hv[i] = hp[idx]; av[i] = ap[idx]; ov[i] = op[idx]; }
        }
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int i = 0; i < NW_MAXV; ++i) {
            const int idx = lane + i * 64;
            if (idx < nv) {
                ss += (hv[i].x * hv[i].x + hv[i].y * hv[i].y) + (hv[i].z * hv[i].z + hv[i].w * hv[i].w);
                dot += (av[i].x * gv[i].x * hv[i].x + av[i].y * gv[i].y * hv[i].y) +
                       (av[i].z * gv[i].z * hv[i].z + av[i].w * gv[i].w * hv[i].w);
            }
        }
        ss = wave_sum(ss);
        dot = wave_sum(dot);
        const float r = rsqrtf(ss / (float)d + eps);
        const float c = r * r * r * dot / (float)d;
        uint2* bp = reinterpret_cast<uint2*>(dhb + (size_t)row * d);
#pragma unroll
        for (int i = 0; i < NW_MAXV; ++i) {
            const int idx = lane + i * 64;
            if (idx < nv) {
                float4 o = ov[i];
                o.x += r * av[i].x * gv[i].x - hv[i].x * c;
                o.y += r * av[i].y * gv[i].y - hv[i].y * c;
                o.z += r * av[i].z * gv[i].z - hv[i].z * c;
                o.w += r * av[i].w * gv[i].w - hv[i].w * c;
                op[idx] = o;
                bp[idx] = make_uint2(pack_bf2(o.x, o.y), pack_bf2(o.z, o.w));
                gacc[i].x += av[i].x * hv[i].x * r;
                gacc[i].y += av[i].y * hv[i].y * r;
                gacc[i].z += av[i].z * hv[i].z * r;
                gacc[i].w += av[i].w * hv[i].w * r;
            }
        }
    }
    // wave 0 stores its partial, waves 1 .. 7 add theirs one after the other: a fixed order
    for (int w = 0; w < NW_WAVES; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < NW_MAXV; ++i) {
                float4 g = gacc[i];
                if (w) {
                    const float4 o = lds[i * 64 + lane];
                    g.x += o.x; g.y += o.y; g.z += o.z; g.w += o.w;
                }
                lds[i * 64 + lane] = g;
            }
        }
        __syncthreads();
    }
    if (wave == 0) {
        float4* pp = reinterpret_cast<float4*>(part + (size_t)blockIdx.x * d);
#pragma unroll
        for (int i = 0; i < NW_MAXV; ++i) {
            const int idx = lane + i * 64;
            if (idx < nv) pp[idx] = lds[i * 64 + lane];
        }
    }
}

__global__ __launch_bounds__(TH) void colsum_final_kernel(const float* __restrict__ part, int nparts, int d,
                                                          float* __restrict__ out) {
    __shared__ float lds[256];
    colsum_rows_body(part, nparts, d, d, out, lds);
}

__global__ __launch_bounds__(TH) void f32_to_bf16_kernel(const float4* __restrict__ src, uint2* __restrict__ dst, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * TH + threadIdx.x; i < n4; i += (size_t)gridDim.x * TH) {
        const float4 v = src[i];
        dst[i] = make_uint2(pack_bf2(v.x, v.y), pack_bf2(v.z, v.w));
    }
}

// delta[b,h,s] = sum_e dO[t, h*hd+e] * O[t, h*hd+e]: one wave per (token, head)
__global__ __launch_bounds__(TH) void attn_delta_kernel(const bf16_t* __restrict__ dO, const bf16_t* __restrict__ O,
                                                        float* __restrict__ delta, int B, int S, int Hq, int hd) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t total = (size_t)B * S * Hq;
    for (size_t it = (size_t)blockIdx.x * 4 + wave; it < total; it += (size_t)gridDim.x * 4) {
        const size_t tok = it / Hq;
        const int hh = (int)(it - tok * Hq);
        const size_t base = tok * (size_t)Hq * hd + (size_t)hh * hd;
        float s = 0.f;
        for (int e = lane * 2; e < hd; e += 128) {
            const uint32_t a = *reinterpret_cast<const uint32_t*>(dO + base + e);
            const uint32_t b = *reinterpret_cast<const uint32_t*>(O + base + e);
            s += bf_lo(a) * bf_lo(b) + bf_hi(a) * bf_hi(b);
        }
        s = wave_sum(s);
        if (lane == 0) {
            const size_t bb = tok / S, ss = tok - bb * S;
            delta[(bb * Hq + hh) * S + ss] = s;
        }
    }
}

inline int grid_for(size_t items, int per_block = TH) {
    size_t g = (items + per_block - 1) / per_block;
    const size_t cap = 256 * 16;
    return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

}  // namespace

hipError_t spk_launch_mse(hipStream_t st, const float* y, const float* t, float* dy, bf16_t* dyb, float* part,
                          float* loss, size_t n) {
    if (n == 0) return hipErrorInvalidValue;
    const int nb = (int)std::min<size_t>(SPK_MSE_PARTS, (n + TH - 1) / TH);
    mse_partial_kernel<<<nb, TH, 0, st>>>(y, t, dy, dyb, part, n, 2.0f / (float)n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    mse_final_kernel<<<1, TH, 0, st>>>(part, nb, loss, 1.0f / (float)n);
    return hipGetLastError();
}

hipError_t spk_launch_swiglu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* gu, int T, int f) {
    if (T <= 0) return hipSuccess;
    if (f <= 0 || (f & 7) || (((uintptr_t)gu | (uintptr_t)dz) & 15)) return hipErrorInvalidValue;
    swiglu_bwd_kernel<<<grid_for((size_t)T * (f >> 3)), TH, 0, st>>>(dz, gu, T, f);
    return hipGetLastError();
}

hipError_t spk_launch_rmsnorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                  bf16_t* dhb, float* part, float* dgain, int T, int d, float eps) {
    if (T <= 0) return hipSuccess;
    if (d <= 0 || (d & 3) || d > TH * NB_MAXV * 4) return hipErrorInvalidValue;
    // which form runs depends on the row length and the row count only
    const bool per_wave = d <= 64 * NW_MAXV * 4 && T >= 4 * SPK_NORM_BWD_BLOCKS;   // enough rows for every wave
    const int nb = per_wave ? SPK_NORM_BWD_BLOCKS : std::min(T, SPK_NORM_BWD_BLOCKS);
    if (per_wave)
        rmsnorm_bwd_wave_kernel<<<nb, NW_WAVES * 64, 0, st>>>(da, h, gain, dh_io, dhb, part, T, d, eps);
    else
        rmsnorm_bwd_kernel<<<nb, TH, 0, st>>>(da, h, gain, dh_io, dhb, part, T, d, eps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    colsum_final_kernel<<<(d + 63) / 64, TH, 0, st>>>(part, nb, d, dgain);
    return hipGetLastError();
}

hipError_t spk_launch_f32_to_bf16(hipStream_t st, const float* src, bf16_t* dst, size_t n) {
    if (n == 0) return hipSuccess;
    if ((n & 3) || (((uintptr_t)src | (uintptr_t)dst) & 15)) return hipErrorInvalidValue;
    f32_to_bf16_kernel<<<grid_for(n >> 2), TH, 0, st>>>(reinterpret_cast<const float4*>(src),
                                                        reinterpret_cast<uint2*>(dst), n >> 2);
    return hipGetLastError();
}

hipError_t spk_launch_attn_delta(hipStream_t st, const bf16_t* dO, const bf16_t* O, float* delta, int B, int S,
                                 int Hq, int hd) {
    if (B <= 0 || S <= 0) return hipSuccess;
    if (hd & 1) return hipErrorInvalidValue;
    attn_delta_kernel<<<grid_for((size_t)B * S * Hq, 4), TH, 0, st>>>(dO, O, delta, B, S, Hq, hd);
    return hipGetLastError();
}
