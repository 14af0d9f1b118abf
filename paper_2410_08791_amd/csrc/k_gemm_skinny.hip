// GEMM for at most 64 activation rows (a decode step: one token per sequence; the ragged last
// rows of a long launch), both operands contraction-contiguous:
// C[M,N] = epilogue(sum_k A(m,k) W(n,k)),  M <= 64.
//
// With so few rows the weight matrix is read once and nothing of it is re-used: the kernel is
// bound by how fast W streams from HBM, and the 256-row tiles of the large kernels leave most of
// the chip without work (N / 128 work-groups, one k-tile in flight each).  Here a work-group owns
// 16 output columns, 16 * MT activation rows and the whole contraction, split over its 8 waves; a
// wave issues its loads straight from global memory, eight k-steps (8 x 1 KiB of W) in flight, and
// contracts with v_mfma_f32_16x16x32_bf16: W rows as the A operand, 16 tokens as the B operand
// (MT such token tiles per W fragment), so a lane ends up with four consecutive output columns of
// one token per tile.  The eight partial results are summed through LDS in wave order
// (deterministic) by wave 0, which applies the epilogue.
//
// More than 16 rows can be taken two ways: MT token tiles in one work-group (every W fragment
// fetched once, N / 16 work-groups), or slices of 16 * MT rows in work-groups of their own.  The
// slices of one column block sit next to each other in the dispatch order and on the same XCD, so
// all but the first find the block in that XCD's L2 (counters: HBM reads are 1.3 x the weight
// bytes with four slices, 1.1 x with one).  One slice is the faster form whenever N / 16 work-groups fill the
// chip; N = 1280 (the ViT-H width) is 80 work-groups, a third of the CUs, and there two slices
// of 32 rows win: 64 x 1280 x 5120 takes 26 -> 17 us, 64 x 1280 x 1280 10 -> 7 us.
// (Measured and not kept: a ring of k-steps re-requested one by one instead of bursts of eight,
// a contraction-index order that uses whole 128-byte lines per step pair, four waves instead of
// eight -- all within 5 % of this form.  With one row tile the kernel streams W at 4.2-5.4 TB/s,
// against 5.7 TB/s for the library's plain row-wise kernels; with 64 rows the L2-to-L1 traffic of
// the re-read activation rows, 4 x the weight bytes, bounds it at ~1.4 TB/s of weights.)
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int SK_WAVES = 8;
constexpr int SK_COLS = 16;     // output columns per work-group

struct SkinnyDev {
    const bf16_t* A; const bf16_t* W; void* C; const float* R; const bf16_t* bias;
    int lda, ldw, ldc, ldr;
    int M, N, K;
    int slices;                 // work-groups per column block; slice i owns rows 16 * MT * i ..
};

// MT: token tiles of 16 rows per work-group
template <int EPI, int MT>
__global__ __launch_bounds__(SK_WAVES * 64) void gemm_skinny_kernel(SkinnyDev p) {
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU_BF16);
    constexpr int NACC = SWIGLU ? 2 : 1;
    // k-steps of 32 whose loads are issued before the first MFMA
    constexpr int SK_UNROLL = MT == 1 ? 8 : MT == 2 ? 6 : 4;
    __shared__ f32x4_t part[NACC][MT][SK_WAVES][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, kb = lane >> 4;
    // dispatch order: groups of 8 column blocks (one per XCD) x slices
    const int per_group = 8 * p.slices;
    const int in_group = blockIdx.x % per_group;
    const int n0 = ((blockIdx.x / per_group) * 8 + (in_group & 7)) * SK_COLS;
    const int m0 = (in_group >> 3) * (16 * MT);
    if (n0 >= p.N) return;       // the last group may be short of column blocks (the whole work-group leaves)

    // this wave's share of the K / 32 contraction steps
    const int steps = p.K / 32;
    const int s0 = (int)((long)steps * wave / SK_WAVES), s1 = (int)((long)steps * (wave + 1) / SK_WAVES);

    // lane (r, kb): row r of the 16-row operand tiles, elements kb*8 .. kb*8+7 of a 32-deep step.
    // Rows past the edge repeat the last valid row; their products land in accumulator rows /
    // columns that are never stored.
    const bf16_t* wp = p.W + (size_t)min(n0 + r, p.N - 1) * p.ldw + kb * 8;
    const bf16_t* wp2 = SWIGLU ? wp + (size_t)p.N * p.ldw : wp;   // the matching "up" rows
    const bf16_t* xp[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) xp[t] = p.A + (size_t)min(m0 + t * 16 + r, p.M - 1) * p.lda + kb * 8;

    f32x4_t acc[NACC][MT];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[a][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    int s = s0;
    for (; s + SK_UNROLL <= s1; s += SK_UNROLL) {
        bf16x8_t wf[NACC][SK_UNROLL], xf[MT][SK_UNROLL];
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u) {
            wf[0][u] = *reinterpret_cast<const bf16x8_t*>(wp + (size_t)(s + u) * 32);
            if (SWIGLU) wf[NACC - 1][u] = *reinterpret_cast<const bf16x8_t*>(wp2 + (size_t)(s + u) * 32);
#pragma unroll
            for (int t = 0; t < MT; ++t) xf[t][u] = *reinterpret_cast<const bf16x8_t*>(xp[t] + (size_t)(s + u) * 32);
        }
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u)
#pragma unroll
            for (int a = 0; a < NACC; ++a)
#pragma unroll
                for (int t = 0; t < MT; ++t)
                    acc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[a][u], xf[t][u], acc[a][t], 0, 0, 0);
    }
    for (; s < s1; ++s) {
        const bf16x8_t w0 = *reinterpret_cast<const bf16x8_t*>(wp + (size_t)s * 32);
        const bf16x8_t w1 = *reinterpret_cast<const bf16x8_t*>(wp2 + (size_t)s * 32);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const bf16x8_t xf = *reinterpret_cast<const bf16x8_t*>(xp[t] + (size_t)s * 32);
            acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, xf, acc[0][t], 0, 0, 0);
            if (SWIGLU) acc[NACC - 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, xf, acc[NACC - 1][t], 0, 0, 0);
        }
    }

#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t) part[a][t][wave][lane] = acc[a][t];
    __syncthreads();
    if (wave != 0) return;

    // accumulator layout of token tile t: lane -> token m = m0 + 16 t + (lane & 15), output
    // columns n0 + 4 * (lane >> 4) + 0..3
    const int n = n0 + 4 * (lane >> 4);
    if (n >= p.N) return;                    // N % 8 == 0: a group of four columns is inside or outside
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = m0 + t * 16 + (lane & 15);
        if (m >= p.M) continue;
        f32x4_t sum[NACC];
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
            sum[a] = part[a][t][0][lane];
#pragma unroll
            for (int w = 1; w < SK_WAVES; ++w) sum[a] += part[a][t][w][lane];
        }
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (SWIGLU) {
                const float gv = sum[0][e], uv = sum[NACC - 1][e];
                v[e] = gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * uv;
            } else {
                v[e] = sum[0][e];
            }
        }
        if (!SWIGLU && p.bias) {
            const uint2 b = *reinterpret_cast<const uint2*>(p.bias + n);
            v[0] += bf_lo(b.x); v[1] += bf_hi(b.x); v[2] += bf_lo(b.y); v[3] += bf_hi(b.y);
        }
        if (EPI == EPI_GELU_BF16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
        }
        if (EPI == EPI_RESID_F32 || EPI == EPI_F32) {
            float4 o = make_float4(v[0], v[1], v[2], v[3]);
            if (EPI == EPI_RESID_F32) {
                const float4 rr = *reinterpret_cast<const float4*>(p.R + (size_t)m * p.ldr + n);
                o = make_float4(o.x + rr.x, o.y + rr.y, o.z + rr.z, o.w + rr.w);
            }
            *reinterpret_cast<float4*>(static_cast<float*>(p.C) + (size_t)m * p.ldc + n) = o;
        } else {
            *reinterpret_cast<uint2*>(static_cast<bf16_t*>(p.C) + (size_t)m * p.ldc + n) =
                make_uint2(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]));
        }
    }
}

// rows_per_group: 0 = chosen here from the shape, else 16, 32 or 64 rows per work-group
template <int EPI>
hipError_t launch_skinny(hipStream_t st, const GemmArgs& g, int rows_per_group) {
    SkinnyDev d;
    d.A = g.A; d.W = g.W; d.C = g.C; d.R = g.R; d.bias = g.bias;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc; d.ldr = g.ldr;
    d.M = g.M; d.N = g.N; d.K = g.K;
    const int col_blocks = (g.N + SK_COLS - 1) / SK_COLS;
    int rpg = rows_per_group;
    if (!rpg) rpg = (g.M > 32 && col_blocks < 128) ? 32 : 64;
    if (rpg > 32 && g.M <= 32) rpg = 32;
    if (rpg > 16 && g.M <= 16) rpg = 16;
    d.slices = (g.M + rpg - 1) / rpg;
    const dim3 grid((col_blocks + 7) / 8 * 8 * d.slices), block(SK_WAVES * 64);
    if (rpg == 16) gemm_skinny_kernel<EPI, 1><<<grid, block, 0, st>>>(d);
    else if (rpg == 32) gemm_skinny_kernel<EPI, 2><<<grid, block, 0, st>>>(d);
    else gemm_skinny_kernel<EPI, 4><<<grid, block, 0, st>>>(d);
    return hipGetLastError();
}

}  // namespace

// Shapes and alignment have been checked by spk_launch_gemm (K % 64 == 0, N % 8 == 0, leading
// dimensions % 8 == 0 resp. % 4 == 0, 16-byte aligned bases); this launcher adds its own limits.
hipError_t spk_launch_gemm_skinny(hipStream_t st, int epi, const GemmArgs& g, int rows_per_group) {
    if (rows_per_group != 0 && rows_per_group != 16 && rows_per_group != 32 && rows_per_group != 64) return hipErrorInvalidValue;
    if (g.M < 1 || g.M > SPK_SKINNY_MAX_ROWS || g.a_form != OP_KMAJOR || g.w_form != OP_KMAJOR) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_BF16: return launch_skinny<EPI_BF16>(st, g, rows_per_group);
        case EPI_RESID_F32: return g.R ? launch_skinny<EPI_RESID_F32>(st, g, rows_per_group) : hipErrorInvalidValue;
        case EPI_GELU_BF16: return g.bias ? launch_skinny<EPI_GELU_BF16>(st, g, rows_per_group) : hipErrorInvalidValue;
        case EPI_SWIGLU_BF16: return !g.bias ? launch_skinny<EPI_SWIGLU_BF16>(st, g, rows_per_group) : hipErrorInvalidValue;
        case EPI_F32: return launch_skinny<EPI_F32>(st, g, rows_per_group);
    }
    return hipErrorInvalidValue;
}
