// Autoregressive decode: key/value cache append and single-query attention over the cache.
//
// Cache of one layer (bf16):  Kt [B][Hkv][hd][max_len]   keys, position index contiguous
//                             V  [B][Hkv][max_len][hd]   values, head dimension contiguous
// Kt is stored transposed so that the score pass reads keys coalesced along the position
// (eight positions per lane); V rows are read coalesced along the head dimension by the
// weighted sum.  Both passes read every cached byte once: the kernel is HBM-bound,
// 4 n Hkv hd bytes per sequence for n cached positions.
#include "sp_common.h"
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
// fp32, weighted sum of V.  Every load is 16 bytes per lane and eight or more are in flight
// per lane: with one work-group per (head, sequence) the kernel is bound by memory latency,
// not bandwidth (4-byte loads four deep took 34 us for 8 x 32 heads over 520 positions).
// Scores: the cache is walked in chunks of 512 positions; a lane owns 8 consecutive positions
// (one 16-byte piece of a Kt row), the four waves split the head dimension, and their partial
// dot products meet in LDS.  Weighted sum: a lane owns 8 consecutive head-dimension elements
// of a V row, a wave 512 / HD rows per step; the partial sums of the waves' row groups meet in
// LDS.  Both reductions add in a fixed order.
// Dynamic LDS (floats): n_pad probabilities | HD query | 8 | 4 x 512 score partials | 2048 output partials.
template <int HD>
__global__ __launch_bounds__(256) void decode_attn_kernel(const bf16_t* __restrict__ qkv, int ld_qkv,
                                                          const bf16_t* __restrict__ kt, const bf16_t* __restrict__ v,
                                                          bf16_t* __restrict__ o, int ld_o, int n, int n_pad,
                                                          int max_len, int Hq, int Hkv, float scale) {
    extern __shared__ float smem[];
    constexpr int DW = HD / 4;             // head-dimension elements per wave in the score pass
    constexpr int LPR = HD / 8;            // lanes per V row
    constexpr int RPW = 64 / LPR;          // V rows per wave and step
    float* sc = smem;
    float* qs = sc + n_pad;
    float* red = qs + HD;
    float* scp = red + 8;                  // [4][512]
    float* part = scp + 4 * 512;           // [4 * RPW][HD]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int hq = blockIdx.x, b = blockIdx.y, hk = hq / (Hq / Hkv);
    if (tid < HD) qs[tid] = bf2f(qkv[(size_t)b * ld_qkv + hq * HD + tid]) * scale;
    __syncthreads();

    // scores.  max_len is a multiple of 8, so a lane's 8 positions lie inside the cache row even
    // when some of them are not among the n valid ones (those are never stored).
    const bf16_t* K = kt + (size_t)(b * Hkv + hk) * HD * max_len + (size_t)w * DW * max_len;
    float mx = -INFINITY;
    for (int c0 = 0; c0 < n; c0 += 512) {
        const int t = c0 + lane * 8;
        float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (t < n) {
            // all of the lane's loads first, then the arithmetic (left to itself the compiler pairs
            // every load with its use and waits for each in turn)
            constexpr int DB = DW < 16 ? DW : 16;
#pragma unroll
            for (int d0 = 0; d0 < DW; d0 += DB) {
                u32x4_t kk[DB];
#pragma unroll
                for (int d = 0; d < DB; ++d) kk[d] = *reinterpret_cast<const u32x4_t*>(K + (size_t)(d0 + d) * max_len + t);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int d = 0; d < DB; ++d) {
                    const float q = qs[w * DW + d0 + d];
                    a[0] = fmaf(q, bf_lo(kk[d][0]), a[0]); a[1] = fmaf(q, bf_hi(kk[d][0]), a[1]);
                    a[2] = fmaf(q, bf_lo(kk[d][1]), a[2]); a[3] = fmaf(q, bf_hi(kk[d][1]), a[3]);
                    a[4] = fmaf(q, bf_lo(kk[d][2]), a[4]); a[5] = fmaf(q, bf_hi(kk[d][2]), a[5]);
                    a[6] = fmaf(q, bf_lo(kk[d][3]), a[6]); a[7] = fmaf(q, bf_hi(kk[d][3]), a[7]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) scp[w * 512 + lane * 8 + e] = a[e];
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = tid * 2 + e;
            if (c0 + i < n) {
                const float sv = (scp[i] + scp[512 + i]) + (scp[1024 + i] + scp[1536 + i]);
                sc[c0 + i] = sv;
                mx = fmaxf(mx, sv);
            }
        }
        __syncthreads();                   // scp is rewritten by the next chunk
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

    // weighted sum: wave w, row group g take keys t = (w * RPW + g) + 4 * RPW * j
    const bf16_t* V = v + (size_t)(b * Hkv + hk) * max_len * HD;
    const int g = lane / LPR, dp = 8 * (lane % LPR);
    float oa[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    constexpr int VB = 8;                  // V rows of a lane in flight
    for (int t0 = w * RPW + g; t0 < n; t0 += VB * 4 * RPW) {
        u32x4_t vv[VB];
        float pr[VB];
#pragma unroll
        for (int j = 0; j < VB; ++j) {
            const int t = t0 + j * 4 * RPW;
            vv[j] = *reinterpret_cast<const u32x4_t*>(V + (size_t)min(t, n - 1) * HD + dp);
            pr[j] = t < n ? sc[t] : 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < VB; ++j) {
            const float p = pr[j];
            oa[0] = fmaf(p, bf_lo(vv[j][0]), oa[0]); oa[1] = fmaf(p, bf_hi(vv[j][0]), oa[1]);
            oa[2] = fmaf(p, bf_lo(vv[j][1]), oa[2]); oa[3] = fmaf(p, bf_hi(vv[j][1]), oa[3]);
            oa[4] = fmaf(p, bf_lo(vv[j][2]), oa[4]); oa[5] = fmaf(p, bf_hi(vv[j][2]), oa[5]);
            oa[6] = fmaf(p, bf_lo(vv[j][3]), oa[6]); oa[7] = fmaf(p, bf_hi(vv[j][3]), oa[7]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[(w * RPW + g) * HD + dp + e] = oa[e];
    __syncthreads();
    if (tid < HD) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4 * RPW; ++i) acc += part[i * HD + tid];
        o[(size_t)b * ld_o + hq * HD + tid] = f2bf(acc / sum);
    }
}

template <int HD>
hipError_t launch_decode(hipStream_t st, const bf16_t* qkv, int ld_qkv, const bf16_t* kt, const bf16_t* v, bf16_t* o,
                         int ld_o, int B, int n, int max_len, int Hq, int Hkv) {
    const int n_pad = (n + 3) / 4 * 4;
    const size_t lds = ((size_t)n_pad + HD + 8 + 4 * 512 + 2048) * sizeof(float);
    static LdsLimitOnce lds_limit;
    if (lds > 48 * 1024) {
        hipError_t e = lds_limit.set(reinterpret_cast<const void*>(decode_attn_kernel<HD>), (int)kDecodeMaxLds);
        if (e != hipSuccess) return e;
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
    if (B < 1 || n < 1 || n > max_len || (max_len & 7) || max_len > kDecodeMaxLen || Hkv < 1 || Hq % Hkv ||
        ((uintptr_t)kt & 15) || ((uintptr_t)v & 15))
        return hipErrorInvalidValue;
    if (hd == 128) return launch_decode<128>(st, qkv, ld_qkv, kt, v, o, ld_o, B, n, max_len, Hq, Hkv);
    if (hd == 64) return launch_decode<64>(st, qkv, ld_qkv, kt, v, o, ld_o, B, n, max_len, Hq, Hkv);
    return hipErrorInvalidValue;
}
