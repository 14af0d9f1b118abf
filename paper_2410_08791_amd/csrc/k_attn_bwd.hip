// Attention backward, two deterministic kernels (no atomics):
//   dq kernel    -- a work-group owns 128 queries of one head and walks the key
//                   tiles, like the forward;
//   dk/dv kernel -- a work-group owns 128 keys of one kv head and walks the
//                   query tiles of every query head that shares it.
// Both recompute P = exp(s - lse) from the forward's log-sum-exp and form
// dS = P * (dP - delta), delta = rowsum(dO * O).
//
// MFMA layouts follow the forward kernel.  In the dq kernel scores are formed
// transposed (S^T = K Q^T, dP^T = V dO^T): a lane holds one query, and dS^T in
// bf16 is already the B operand of dQ^T = K^T dS^T.  In the dk/dv kernel scores
// are formed straight (S = Q K^T, dP = dO V^T): a lane holds one key, and P, dS
// in bf16 are the B operands of dV^T = dO^T P and dK^T = Q^T dS.  The A operands
// K^T, dO^T, Q^T are read out of the same token-row LDS tiles the score products use,
// through the transposing LDS read: no transposed copies exist in memory.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

template <int HD>
struct BwdCfg {
    static constexpr int NKS = HD / 16;
    static constexpr int NMT = (HD + 31) / 32;
};

// Transposed MFMA operand out of a token-row tile (rows = tokens, head dimension contiguous):
// the lane ends up with head-dimension row (lane & 31) of the 32-row block the pointer selects
// and the eight tokens 4*half + {0..3} and 8 + 4*half + {0..3} of a 16-token step -- the token
// order in which the score tiles hold their bf16 operands.  ds_read_b64_tr_b16 works on groups
// of 16 lanes: lane s supplies the address of four values of one token row, lane i receives
// element i%4 of the blocks supplied by lanes i/4, i/4+4, i/4+8, i/4+12.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
__device__ __forceinline__ int tr_lane_off(int lane, int stride) {
    const int s16 = lane & 15, half = lane >> 5;
    return (4 * half + (s16 >> 2)) * stride + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
}
__device__ __forceinline__ bf16x8_t tr_frag_tok(const unsigned char* p, int stride) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 8 * stride));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, both);
}

// Row stride (bytes) of a token-row tile: 16 * odd keeps the 16-byte row reads of the score
// products conflict-free, and the residue spreads the four token rows of a transposed read.
template <int HD> struct TokTile { static constexpr int RS = ((HD + 31) / 32 * 32) * 2 + 48; };
template <> struct TokTile<80> { static constexpr int RS = 96 * 2 + 16; };
template <> struct TokTile<64> { static constexpr int RS = 64 * 2 + 16; };

// ------------------------------------------------------------------------- dq
// A work-group owns 128 queries of one head (a wave 32 of them, one query per lane as the B
// operand) and walks 64-key tiles.  K and V tiles sit in LDS as token rows: S^T = K Q^T and
// dP^T = V dO^T read them straight, dQ^T += K^T dS^T reads K through the transposing LDS
// read.  The next tile's rows are fetched into registers before the current one is computed.
// (Two work-groups per CU: the kernel fits 256 registers at every head dimension.)
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          bf16_t* __restrict__ dqkv, int S, int Hq, int Hkv, int ld_qkv,
                                                          int causal, float scale, float scale_log2e) {
    typedef BwdCfg<HD> C;
    constexpr int KB = 64, RS = TokTile<HD>::RS;
    constexpr int CHUNKS = KB * (HD / 8), ITERS = (CHUNKS + 255) / 256;
    __shared__ __attribute__((aligned(16))) unsigned char sK[KB * RS];
    __shared__ __attribute__((aligned(16))) unsigned char sV[KB * RS];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    // work-group ids are dealt round-robin to the 8 XCDs: remapped so that an XCD works through a
    // contiguous range of (batch, head, query block) and a head's keys and values are fetched
    // through one L2
    const int job = xcd_remap(blockIdx.x + (int)gridDim.x * (blockIdx.y + (int)gridDim.y * blockIdx.z),
                              (int)(gridDim.x * gridDim.y * gridDim.z));
    const int bx = job % (int)gridDim.x, h = (job / (int)gridDim.x) % (int)gridDim.y, b = job / (int)(gridDim.x * gridDim.y);
    const int qb = causal ? gridDim.x - 1 - bx : bx;
    const int kvh = h / (Hq / Hkv);
    const int q0 = qb * 128, wq0 = q0 + wave * 32, qi = wq0 + l32;
    const size_t tok0 = (size_t)b * S;
    const int qr = min(qi, S - 1);

    bf16x8_t qf[C::NKS], dof[C::NKS];
    {
        const bf16_t* qp = qkv + (tok0 + qr) * ld_qkv + h * HD + half * 8;
        const bf16_t* dp = dO + (tok0 + qr) * (size_t)(Hq * HD) + h * HD + half * 8;
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) {
            qf[ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16);
            dof[ks] = *reinterpret_cast<const bf16x8_t*>(dp + ks * 16);
        }
    }
    const float lse_q = lse[((size_t)b * Hq + h) * S + qr] * 1.4426950408889634f;
    const float delta_q = delta[((size_t)b * Hq + h) * S + qr];
    const bf16_t* kbase = qkv + tok0 * ld_qkv + (size_t)Hq * HD + (size_t)kvh * HD;
    const bf16_t* vbase = kbase + (size_t)Hkv * HD;
    const int tro = tr_lane_off(lane, RS);

    f32x16_t acc[C::NMT];
#pragma unroll
    for (int t = 0; t < C::NMT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    u32x4_t rk[ITERS], rv[ITERS];
    auto fetch = [&](int tile) {
        const int key0 = tile * KB;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int c = threadIdx.x + i * 256;
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
                const int r = c / (HD / 8), cc = c % (HD / 8);
                const size_t row = (size_t)min(key0 + r, S - 1) * ld_qkv + cc * 8;
                rk[i] = *reinterpret_cast<const u32x4_t*>(kbase + row);
                rv[i] = *reinterpret_cast<const u32x4_t*>(vbase + row);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int c = threadIdx.x + i * 256;
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
                const int r = c / (HD / 8), cc = c % (HD / 8);
                *reinterpret_cast<u32x4_t*>(sK + r * RS + cc * 16) = rk[i];
                *reinterpret_cast<u32x4_t*>(sV + r * RS + cc * 16) = rv[i];
            }
        }
    };

    const int k_end = causal ? min(S, q0 + 128) : S;
    const int ntiles = (k_end + KB - 1) / KB;
    fetch(0);
    for (int tile = 0; tile < ntiles; ++tile) {
        const int key0 = tile * KB;
        __syncthreads();
        stash();
        __syncthreads();
        if (tile + 1 < ntiles) fetch(tile + 1);
        if (causal && key0 > wq0 + 31) continue;

        bf16x8_t dsf[2][2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x16_t s, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < C::NKS; ++ks) {
                const int off = (t * 32 + l32) * RS + (ks * 2 + half) * 16;
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(sK + off), qf[ks], s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(sV + off), dof[ks], dp, 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = key0 + t * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                const bool ok = key < S && (!causal || key <= qi);
                const float p = ok ? __builtin_amdgcn_exp2f(fmaf(s[e], scale_log2e, -lse_q)) : 0.f;
                dsf[t][e >> 3][e & 7] = (__bf16)(p * (dp[e] - delta_q));
            }
        }
#pragma unroll
        for (int mt = 0; mt < C::NMT; ++mt)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        tr_frag_tok(sK + (t * 32 + 16 * j) * RS + mt * 64 + tro, RS), dsf[t][j], acc[mt], 0, 0, 0);
    }
    if (qi < S) {
        bf16_t* op = dqkv + (tok0 + qi) * ld_qkv + h * HD;
#pragma unroll
        for (int mt = 0; mt < C::NMT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e0 = mt * 32 + g * 8 + half * 4;
                if (e0 < HD)
                    *reinterpret_cast<uint2*>(op + e0) =
                        make_uint2(pack_bf2(acc[mt][g * 4] * scale, acc[mt][g * 4 + 1] * scale),
                                   pack_bf2(acc[mt][g * 4 + 2] * scale, acc[mt][g * 4 + 3] * scale));
            }
    }
}

// ---------------------------------------------------------------------- dk, dv
// A work-group owns 128 keys of one kv head (a wave 32 of them, one key per lane as the B
// operand of S = Q K^T and dP = dO V^T) and walks 64-query tiles of every query head of the
// group.  Q and dO tiles sit in LDS once, as token rows: the score products read them
// straight, dV^T += dO^T P and dK^T += Q^T dS read them through the transposing LDS read.
// The next tile's rows are fetched into registers before the current tile is computed.
// At head_dim 128 a wave holds dK^T and dV^T of its 32 keys (128 registers), its K and V
// fragments (64) and the score / dP tiles: ~370 registers, one wave per SIMD; the smaller head
// dimensions fit two.
template <int HD>
__global__ __launch_bounds__(256, HD <= 80 ? 2 : 1) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, int S, int Hq, int Hkv,
                                                           int ld_qkv, int causal, float scale, float scale_log2e) {
    typedef BwdCfg<HD> C;
    constexpr int QT = 64, RS = TokTile<HD>::RS;
    constexpr int CHUNKS = QT * (HD / 8), ITERS = (CHUNKS + 255) / 256;
    __shared__ __attribute__((aligned(16))) unsigned char sQ[QT * RS];
    __shared__ __attribute__((aligned(16))) unsigned char sdO[QT * RS];
    __shared__ float s_lse[QT], s_delta[QT];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    // the same XCD-contiguous order as in the dq kernel: the key blocks of a head share its queries
    const int job = xcd_remap(blockIdx.x + (int)gridDim.x * (blockIdx.y + (int)gridDim.y * blockIdx.z),
                              (int)(gridDim.x * gridDim.y * gridDim.z));
    const int bx = job % (int)gridDim.x, kvh = (job / (int)gridDim.x) % (int)gridDim.y, b = job / (int)(gridDim.x * gridDim.y);
    const int grp = Hq / Hkv;
    const int k0 = bx * 128, wk0 = k0 + wave * 32, kj = wk0 + l32;
    const size_t tok0 = (size_t)b * S;
    const int ld_do = Hq * HD;

    bf16x8_t kf[C::NKS], vf[C::NKS];
    {
        const bf16_t* kp = qkv + (tok0 + min(kj, S - 1)) * ld_qkv + (size_t)Hq * HD + (size_t)kvh * HD + half * 8;
        const bf16_t* vp = kp + (size_t)Hkv * HD;
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) {
            kf[ks] = *reinterpret_cast<const bf16x8_t*>(kp + ks * 16);
            vf[ks] = *reinterpret_cast<const bf16x8_t*>(vp + ks * 16);
        }
    }
    f32x16_t dk[C::NMT], dv[C::NMT];
#pragma unroll
    for (int t = 0; t < C::NMT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dk[t][e] = 0.f; dv[t][e] = 0.f; }

    // the tiles of this work-group in walking order: (query head of the group, 64-query tile)
    const int q_begin = causal ? (k0 / QT) * QT : 0;
    const int tiles_per_head = (S - q_begin + QT - 1) / QT;
    const int n_tiles = grp * tiles_per_head;
    const int tro = tr_lane_off(lane, RS);

    u32x4_t rq[ITERS], rdo[ITERS];
    float r_lse = 0.f, r_delta = 0.f;
    auto fetch = [&](int tile) {
        const int h = kvh * grp + tile / tiles_per_head;
        const int q0 = q_begin + (tile % tiles_per_head) * QT;
        const bf16_t* qbase = qkv + tok0 * ld_qkv + h * HD;
        const bf16_t* dobase = dO + tok0 * (size_t)ld_do + h * HD;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int c = threadIdx.x + i * 256;
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
                const int r = c / (HD / 8), cc = c % (HD / 8);
                const int row = min(q0 + r, S - 1);
                rq[i] = *reinterpret_cast<const u32x4_t*>(qbase + (size_t)row * ld_qkv + cc * 8);
                rdo[i] = *reinterpret_cast<const u32x4_t*>(dobase + (size_t)row * ld_do + cc * 8);
            }
        }
        if (threadIdx.x < QT) {
            const int row = min(q0 + (int)threadIdx.x, S - 1);
            r_lse = lse[((size_t)b * Hq + h) * S + row] * 1.4426950408889634f;
            r_delta = delta[((size_t)b * Hq + h) * S + row];
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int c = threadIdx.x + i * 256;
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
                const int r = c / (HD / 8), cc = c % (HD / 8);
                *reinterpret_cast<u32x4_t*>(sQ + r * RS + cc * 16) = rq[i];
                *reinterpret_cast<u32x4_t*>(sdO + r * RS + cc * 16) = rdo[i];
            }
        }
        if (threadIdx.x < QT) { s_lse[threadIdx.x] = r_lse; s_delta[threadIdx.x] = r_delta; }
    };

    if (n_tiles > 0) fetch(0);
    for (int tile = 0; tile < n_tiles; ++tile) {
        __syncthreads();                      // everyone is done reading the previous tile
        stash();
        __syncthreads();
        if (tile + 1 < n_tiles) fetch(tile + 1);
        const int q0 = q_begin + (tile % tiles_per_head) * QT;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int qs = q0 + sub * 32;
            if (qs >= S) continue;
            if (causal && qs + 31 < wk0) continue;   // every query of the sub-tile precedes this wave's keys
            f32x16_t s, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < C::NKS; ++ks) {
                const int off = (sub * 32 + l32) * RS + (ks * 2 + half) * 16;
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(sQ + off), kf[ks], s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(sdO + off), vf[ks], dp, 0, 0, 0);
            }
            bf16x8_t pf[2], dsf[2];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = (e >> 2) * 8 + half * 4 + (e & 3);
                const int q = qs + r;
                const bool ok = q < S && (!causal || kj <= q);
                const float p = ok ? __builtin_amdgcn_exp2f(fmaf(s[e], scale_log2e, -s_lse[sub * 32 + r])) : 0.f;
                pf[e >> 3][e & 7] = (__bf16)p;
                dsf[e >> 3][e & 7] = (__bf16)(p * (dp[e] - s_delta[sub * 32 + r]));
            }
#pragma unroll
            for (int mt = 0; mt < C::NMT; ++mt)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int off = (sub * 32 + 16 * j) * RS + mt * 64 + tro;
                    dv[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag_tok(sdO + off, RS), pf[j], dv[mt], 0, 0, 0);
                    dk[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag_tok(sQ + off, RS), dsf[j], dk[mt], 0, 0, 0);
                }
        }
    }
    if (kj < S) {
        bf16_t* kp = dqkv + (tok0 + kj) * ld_qkv + (size_t)Hq * HD + (size_t)kvh * HD;
        bf16_t* vp = kp + (size_t)Hkv * HD;
#pragma unroll
        for (int mt = 0; mt < C::NMT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e0 = mt * 32 + g * 8 + half * 4;
                if (e0 < HD) {
                    *reinterpret_cast<uint2*>(kp + e0) =
                        make_uint2(pack_bf2(dk[mt][g * 4] * scale, dk[mt][g * 4 + 1] * scale),
                                   pack_bf2(dk[mt][g * 4 + 2] * scale, dk[mt][g * 4 + 3] * scale));
                    *reinterpret_cast<uint2*>(vp + e0) =
                        make_uint2(pack_bf2(dv[mt][g * 4], dv[mt][g * 4 + 1]), pack_bf2(dv[mt][g * 4 + 2], dv[mt][g * 4 + 3]));
                }
            }
    }
}

template <int HD>
hipError_t launch_bwd(hipStream_t st, const AttnBwdArgs& g, const AttnShape& a) {
    const float scale = 1.0f / sqrtf((float)a.hd), sl2 = scale * 1.4426950408889634f;
    dim3 gq((a.S + 127) / 128, a.Hq, a.B);
    attn_bwd_dq_kernel<HD><<<gq, 256, 0, st>>>(g.qkv, g.dO, g.lse, g.delta, g.dqkv, a.S, a.Hq, a.Hkv, a.ld_qkv, a.causal,
                                               scale, sl2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 gk((a.S + 127) / 128, a.Hkv, a.B);
    attn_bwd_dkv_kernel<HD><<<gk, 256, 0, st>>>(g.qkv, g.dO, g.lse, g.delta, g.dqkv, a.S, a.Hq, a.Hkv, a.ld_qkv,
                                                a.causal, scale, sl2);
    return hipGetLastError();
}

}  // namespace

hipError_t spk_launch_attention_bwd(hipStream_t st, const AttnBwdArgs& g, const AttnShape& a) {
    if (a.B <= 0 || a.S <= 0) return hipSuccess;
    if (a.Hkv <= 0 || a.Hq % a.Hkv || a.ld_qkv % 8 || a.B > 65535 || a.Hq > 65535) return hipErrorInvalidValue;
    if (!g.qkv || !g.dO || !g.lse || !g.delta || !g.dqkv) return hipErrorInvalidValue;
    switch (a.hd) {
        case 64: return launch_bwd<64>(st, g, a);
        case 80: return launch_bwd<80>(st, g, a);
        case 128: return launch_bwd<128>(st, g, a);
    }
    return hipErrorInvalidValue;
}
