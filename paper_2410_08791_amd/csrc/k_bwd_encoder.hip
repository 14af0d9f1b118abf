// Backward kernels that only the encoder layer needs: LayerNorm backward (gain and
// bias gradients by the same deterministic two-stage reduction as RMSNorm), GELU and its
// backward as element-wise passes, and column sums over tokens for the bias gradients of
// the linear maps.  All HBM-bound: each reads and writes its operands once.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int TH = 256;
constexpr int LN_MAXV = 8;   // float4 per thread -> d <= 8192

// a = (h - mean) r g + b, r = rsqrt(var + eps) (biased variance).  Given da:
//   xhat = (h - mean) r,  q = da g,
//   dh_io += r (q - mean(q) - xhat mean(q xhat)),  dgain = sum_t da xhat,  dbias = sum_t da.
// Block b owns rows b, b+G, ...; partial row b of `part` = [dgain | dbias] of those rows.
__global__ __launch_bounds__(TH) void layernorm_bwd_kernel(const float* __restrict__ da, const float* __restrict__ h,
                                                           const bf16_t* __restrict__ gain, float* __restrict__ dh_io,
                                                           bf16_t* __restrict__ dhb, float* __restrict__ part, int T,
                                                           int d, float eps) {
    __shared__ float red[8];
    const int nv = d >> 2;
    const float inv_d = 1.0f / (float)d;
    float4 gacc[LN_MAXV], bacc[LN_MAXV], gv[LN_MAXV];
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        gacc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        bacc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        const int idx = threadIdx.x + i * TH;
        if (idx < nv) {
            const uint2 g = reinterpret_cast<const uint2*>(gain)[idx];
            gv[i] = make_float4(bf_lo(g.x), bf_hi(g.x), bf_lo(g.y), bf_hi(g.y));
        }
    }
    for (int row = blockIdx.x; row < T; row += gridDim.x) {
        const float4* hp = reinterpret_cast<const float4*>(h + (size_t)row * d);
        const float4* ap = reinterpret_cast<const float4*>(da + (size_t)row * d);
        float4 hv[LN_MAXV], av[LN_MAXV];
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                hv[i] = hp[idx];
                av[i] = ap[idx];
                s += (hv[i].x + hv[i].y) + (hv[i].z + hv[i].w);
            }
        }
        const float mean = block_sum_256(s, red) * inv_d;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                hv[i].x -= mean; hv[i].y -= mean; hv[i].z -= mean; hv[i].w -= mean;
                ss += (hv[i].x * hv[i].x + hv[i].y * hv[i].y) + (hv[i].z * hv[i].z + hv[i].w * hv[i].w);
            }
        }
        const float r = rsqrtf(block_sum_256(ss, red + 4) * inv_d + eps);
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                hv[i].x *= r; hv[i].y *= r; hv[i].z *= r; hv[i].w *= r;          // xhat
                const float qx = av[i].x * gv[i].x, qy = av[i].y * gv[i].y, qz = av[i].z * gv[i].z,
                            qw = av[i].w * gv[i].w;
                s1 += (qx + qy) + (qz + qw);
                s2 += (qx * hv[i].x + qy * hv[i].y) + (qz * hv[i].z + qw * hv[i].w);
            }
        }
        const float m1 = block_sum_256(s1, red) * inv_d;
        const float m2 = block_sum_256(s2, red + 4) * inv_d;
        float4* op = reinterpret_cast<float4*>(dh_io + (size_t)row * d);
        uint2* bp = reinterpret_cast<uint2*>(dhb + (size_t)row * d);
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) {
            const int idx = threadIdx.x + i * TH;
            if (idx < nv) {
                float4 o = op[idx];
                o.x += r * (av[i].x * gv[i].x - m1 - hv[i].x * m2);
                o.y += r * (av[i].y * gv[i].y - m1 - hv[i].y * m2);
                o.z += r * (av[i].z * gv[i].z - m1 - hv[i].z * m2);
                o.w += r * (av[i].w * gv[i].w - m1 - hv[i].w * m2);
                op[idx] = o;
                bp[idx] = make_uint2(pack_bf2(o.x, o.y), pack_bf2(o.z, o.w));
                gacc[i].x += av[i].x * hv[i].x; gacc[i].y += av[i].y * hv[i].y;
                gacc[i].z += av[i].z * hv[i].z; gacc[i].w += av[i].w * hv[i].w;
                bacc[i].x += av[i].x; bacc[i].y += av[i].y; bacc[i].z += av[i].z; bacc[i].w += av[i].w;
            }
        }
    }
    float4* pg = reinterpret_cast<float4*>(part + (size_t)blockIdx.x * 2 * d);
    float4* pb = reinterpret_cast<float4*>(part + (size_t)blockIdx.x * 2 * d + d);
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int idx = threadIdx.x + i * TH;
        if (idx < nv) { pg[idx] = gacc[i]; pb[idx] = bacc[i]; }
    }
}

__global__ __launch_bounds__(TH) void colsum_rows_kernel(const float* __restrict__ part, int nparts, int ld, int n,
                                                         float* __restrict__ out) {
    __shared__ float lds[256];
    colsum_rows_body(part, nparts, ld, n, out, lds);
}

// z = gelu(u), 8 elements per thread
__global__ __launch_bounds__(TH) void gelu_kernel(const bf16_t* __restrict__ u, bf16_t* __restrict__ z, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * TH + threadIdx.x; i < n8; i += (size_t)gridDim.x * TH) {
        const u32x4_t v = reinterpret_cast<const u32x4_t*>(u)[i];
        u32x4_t o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = pack_bf2(gelu_erf(bf_lo(v[k])), gelu_erf(bf_hi(v[k])));
        reinterpret_cast<u32x4_t*>(z)[i] = o;
    }
}

// u <- dz * gelu'(u), in place over the pre-activation
__global__ __launch_bounds__(TH) void gelu_bwd_kernel(const bf16_t* __restrict__ dz, bf16_t* __restrict__ u, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * TH + threadIdx.x; i < n8; i += (size_t)gridDim.x * TH) {
        const u32x4_t v = reinterpret_cast<const u32x4_t*>(u)[i];
        const u32x4_t g = reinterpret_cast<const u32x4_t*>(dz)[i];
        u32x4_t o;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            o[k] = pack_bf2(bf_lo(g[k]) * gelu_erf_grad(bf_lo(v[k])), bf_hi(g[k]) * gelu_erf_grad(bf_hi(v[k])));
        reinterpret_cast<u32x4_t*>(u)[i] = o;
    }
}

// part[b][c] = sum of src[row][c] over rows b, b+G, ...  (src bf16 [T, ld], n columns)
__global__ __launch_bounds__(TH) void colsum_bf16_kernel(const bf16_t* __restrict__ src, int ld, int T, int n,
                                                         float* __restrict__ part) {
    for (int c = 2 * threadIdx.x; c < n; c += 2 * TH) {
        float s0 = 0.f, s1 = 0.f;
        for (int row = blockIdx.x; row < T; row += gridDim.x) {
            const uint32_t v = *reinterpret_cast<const uint32_t*>(src + (size_t)row * ld + c);
            s0 += bf_lo(v);
            s1 += bf_hi(v);
        }
        part[(size_t)blockIdx.x * n + c] = s0;
        part[(size_t)blockIdx.x * n + c + 1] = s1;
    }
}

inline int grid_for(size_t items) {
    size_t g = (items + TH - 1) / TH;
    const size_t cap = 256 * 16;
    return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

}  // namespace

hipError_t spk_launch_layernorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                    bf16_t* dhb, float* part, float* dgain, float* dbias, int T, int d, float eps) {
    if (T <= 0) return hipSuccess;
    if (d <= 0 || (d & 3) || d > TH * LN_MAXV * 4) return hipErrorInvalidValue;
    const int nb = std::min(T, SPK_NORM_BWD_BLOCKS);
    layernorm_bwd_kernel<<<nb, TH, 0, st>>>(da, h, gain, dh_io, dhb, part, T, d, eps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    colsum_rows_kernel<<<(d + 63) / 64, TH, 0, st>>>(part, nb, 2 * d, d, dgain);
    colsum_rows_kernel<<<(d + 63) / 64, TH, 0, st>>>(part + d, nb, 2 * d, d, dbias);
    return hipGetLastError();
}

hipError_t spk_launch_gelu(hipStream_t st, const bf16_t* u, bf16_t* z, size_t n) {
    if (n == 0) return hipSuccess;
    if ((n & 7) || (((uintptr_t)u | (uintptr_t)z) & 15)) return hipErrorInvalidValue;
    gelu_kernel<<<grid_for(n >> 3), TH, 0, st>>>(u, z, n >> 3);
    return hipGetLastError();
}

hipError_t spk_launch_gelu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* u, size_t n) {
    if (n == 0) return hipSuccess;
    if ((n & 7) || (((uintptr_t)u | (uintptr_t)dz) & 15)) return hipErrorInvalidValue;
    gelu_bwd_kernel<<<grid_for(n >> 3), TH, 0, st>>>(dz, u, n >> 3);
    return hipGetLastError();
}

hipError_t spk_launch_colsum_bf16(hipStream_t st, const bf16_t* src, int ld, int T, int n, float* part, float* out) {
    if (T <= 0 || n <= 0) return hipSuccess;
    if ((n & 1) || (ld & 1) || ((uintptr_t)src & 3)) return hipErrorInvalidValue;
    const int nb = std::min(T, SPK_NORM_BWD_BLOCKS);
    colsum_bf16_kernel<<<nb, TH, 0, st>>>(src, ld, T, n, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    colsum_rows_kernel<<<(n + 63) / 64, TH, 0, st>>>(part, nb, n, n, out);
    return hipGetLastError();
}
