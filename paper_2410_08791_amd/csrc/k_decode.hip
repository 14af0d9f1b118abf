// Autoregressive decode: key/value cache append and single-query attention over the cache.
//
// Cache of one layer (bf16):  Kt [B][Hkv][hd][max_len]   keys, position index contiguous
//                             V  [B][Hkv][max_len][hd]   values, head dimension contiguous
// Kt is stored transposed so that the score pass reads keys coalesced along the position
// (one lane per key pair); V rows are read coalesced along the head dimension by the
// weighted sum.  Both passes read every cached byte once: the kernel is HBM-bound,
// 4 n Hkv hd bytes per sequence for n cached positions.
#include "sp_kernels.h"

namespace {

// Append S new positions (pos0 .. pos0+S-1) of every sequence from the fused activation
// qkv [B*S, ld] = [q | k | v].  One work-group: 64 positions of one (batch, kv head).
__global__ __launch_bounds__(256) void kv_append_kernel(const bf16_t* __restrict__ qkv, int ld, bf16_t* __restrict__ kt,
                                                        bf16_t* __restrict__ v, int S, int pos0, int Hq, int Hkv,
                                                        int hd, int max_len) {
    __shared__ bf16_t tile[64][130];
    const int s0 = blockIdx.x * 64, h = blockIdx.y, b = blockIdx.z;
    const int ns = min(64, S - s0);
    const bf16_t* ksrc = qkv + (size_t)(b * S + s0) * ld + (size_t)(Hq + h) * hd;
    const bf16_t* vsrc = ksrc + (size_t)Hkv * hd;
    bf16_t* vdst = v + ((size_t)(b * Hkv + h) * max_len + pos0 + s0) * hd;
    for (int i = threadIdx.x; i < ns * hd; i += 256) {
        const int s = i / hd, d = i - s * hd;
        tile[s][d] = ksrc[(size_t)s * ld + d];
        vdst[(size_t)s * hd + d] = vsrc[(size_t)s * ld + d];
    }
    __syncthreads();
    bf16_t* kdst = kt + (size_t)(b * Hkv + h) * hd * max_len + pos0 + s0;
    const int s = threadIdx.x & 63;
    if (s < ns)
        for (int d = threadIdx.x >> 6; d < hd; d += 4) kdst[(size_t)d * max_len + s] = tile[s][d];
}

// One work-group = one (query head, sequence): scores over n cached positions, softmax in
// fp32, weighted sum of V.  Dynamic LDS: n_pad scores | HD query | 8 | 4*KPW*HD partial sums.
template <int HD>
__global__ __launch_bounds__(256) void decode_attn_kernel(const bf16_t* __restrict__ qkv, int ld_qkv,
                                                          const bf16_t* __restrict__ kt, const bf16_t* __restrict__ v,
                                                          bf16_t* __restrict__ o, int ld_o, int n, int n_pad,
                                                          int max_len, int Hq, int Hkv, float scale) {
    extern __shared__ float smem[];
    constexpr int KPW = 128 / HD;          // keys one wave handles per step of the weighted sum
    float* sc = smem;
    float* qs = sc + n_pad;
    float* red = qs + HD;
    float* part = red + 8;                 // [4 * KPW][HD]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int hq = blockIdx.x, b = blockIdx.y, hk = hq / (Hq / Hkv);
    if (tid < HD) qs[tid] = bf2f(qkv[(size_t)b * ld_qkv + hq * HD + tid]) * scale;
    __syncthreads();

    // scores: a thread owns key pairs (t, t+1), t = 2*tid + 512*j; max_len is even, so the
    // pair's second key is inside the cache even when it is not among the n valid ones
    const bf16_t* K = kt + (size_t)(b * Hkv + hk) * HD * max_len;
    float mx = -INFINITY;
    for (int t = 2 * tid; t < n; t += 512) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll 16
        for (int d = 0; d < HD; ++d) {
            const uint32_t kk = *reinterpret_cast<const uint32_t*>(K + (size_t)d * max_len + t);
            a0 = fmaf(qs[d], bf_lo(kk), a0);
            a1 = fmaf(qs[d], bf_hi(kk), a1);
        }
        sc[t] = a0;
        mx = fmaxf(mx, a0);
        if (t + 1 < n) { sc[t + 1] = a1; mx = fmaxf(mx, a1); }
    }
    mx = wave_max(mx);
    if (lane == 0) red[w] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.f;
    for (int t = tid; t < n; t += 256) {
        const float p = __expf(sc[t] - mx);
        sc[t] = p;
        sum += p;
    }
    sum = block_sum_256(sum, red + 4);     // its barriers also publish the probabilities

    // weighted sum: wave w, sub-group g take keys t = (w*KPW + g) + 4*KPW*j; a lane holds two
    // adjacent head-dimension elements
    const bf16_t* V = v + (size_t)(b * Hkv + hk) * max_len * HD;
    const int g = lane / (HD / 2), dp = 2 * (lane % (HD / 2));
    float o0 = 0.f, o1 = 0.f;
#pragma unroll 4
    for (int t = w * KPW + g; t < n; t += 4 * KPW) {
        const uint32_t vv = *reinterpret_cast<const uint32_t*>(V + (size_t)t * HD + dp);
        const float p = sc[t];
        o0 = fmaf(p, bf_lo(vv), o0);
        o1 = fmaf(p, bf_hi(vv), o1);
    }
    part[(w * KPW + g) * HD + dp] = o0;
    part[(w * KPW + g) * HD + dp + 1] = o1;
    __syncthreads();
    if (tid < HD) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4 * KPW; ++i) acc += part[i * HD + tid];
        o[(size_t)b * ld_o + hq * HD + tid] = f2bf(acc / sum);
    }
}

template <int HD>
hipError_t launch_decode(hipStream_t st, const bf16_t* qkv, int ld_qkv, const bf16_t* kt, const bf16_t* v, bf16_t* o,
                         int ld_o, int B, int n, int max_len, int Hq, int Hkv) {
    const int n_pad = (n + 3) / 4 * 4;
    const size_t lds = ((size_t)n_pad + HD + 8 + 4 * (128 / HD) * HD) * sizeof(float);
    static size_t attr = 0;
    if (lds > 48 * 1024 && lds > attr) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_attn_kernel<HD>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDecodeMaxLds);
        if (e != hipSuccess) return e;
        attr = kDecodeMaxLds;
    }
    decode_attn_kernel<HD><<<dim3(Hq, B), 256, lds, st>>>(qkv, ld_qkv, kt, v, o, ld_o, n, n_pad, max_len, Hq, Hkv,
                                                          1.0f / sqrtf((float)HD));
    return hipGetLastError();
}

}  // namespace

hipError_t spk_launch_kv_append(hipStream_t st, const bf16_t* qkv, int ld_qkv, bf16_t* kt, bf16_t* v, int B, int S,
                                int pos0, int Hq, int Hkv, int hd, int max_len) {
    if (B < 1 || S < 1 || pos0 < 0 || pos0 + S > max_len || hd > 128 || hd < 1 || Hkv < 1 || Hq < Hkv)
        return hipErrorInvalidValue;
    kv_append_kernel<<<dim3((S + 63) / 64, Hkv, B), 256, 0, st>>>(qkv, ld_qkv, kt, v, S, pos0, Hq, Hkv, hd, max_len);
    return hipGetLastError();
}

hipError_t spk_launch_decode_attention(hipStream_t st, const bf16_t* qkv, int ld_qkv, const bf16_t* kt,
                                       const bf16_t* v, bf16_t* o, int ld_o, int B, int n, int max_len, int Hq,
                                       int Hkv, int hd) {
    if (B < 1 || n < 1 || n > max_len || (max_len & 1) || max_len > kDecodeMaxLen || Hkv < 1 || Hq % Hkv ||
        ((uintptr_t)kt & 3) || ((uintptr_t)v & 3))
        return hipErrorInvalidValue;
    if (hd == 128) return launch_decode<128>(st, qkv, ld_qkv, kt, v, o, ld_o, B, n, max_len, Hq, Hkv);
    if (hd == 64) return launch_decode<64>(st, qkv, ld_qkv, kt, v, o, ld_o, B, n, max_len, Hq, Hkv);
    return hipErrorInvalidValue;
}
