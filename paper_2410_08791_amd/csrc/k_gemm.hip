// bf16 GEMM on the gfx950 matrix cores: C[M,N] = sum_k A(m,k) W(n,k), fp32
// accumulate, used for every dense projection of a layer (QKV, O, gate/up,
// down) and for the backward contractions.
//
// Work-group = 4 or 8 waves in a 2 x (waves/2) grid; block tile BM x BN x 64,
// each wave owns its share as 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16).
// Both operand tiles are staged in LDS with the contraction index contiguous
// (128-byte rows, 16-byte chunks XOR-swizzled so that both the 16-byte stores
// and the per-lane 16-byte fragment loads spread over all banks), double
// buffered.  Two kernels build that LDS image: gemm_dma_kernel (global loads
// that write LDS directly; used whenever both operands have the contraction
// index contiguous, i.e. every forward projection) and gemm_kernel (register
// staging: global loads for tile t+1 are issued before the MFMAs of tile t and
// stored to the other buffer afterwards, one barrier per tile; takes every
// operand form).
//
// The MFMA is issued "transposed" (weights as the A operand, activations as B)
// so that a lane's four consecutive accumulator registers are four consecutive
// n of one row m: the epilogue then writes 8-byte (bf16) or 16-byte (fp32)
// pieces of a row instead of single elements.
//
// An operand whose contraction index is NOT contiguous in memory (the backward
// GEMMs) is staged as it lies in memory (LDS row = contraction index) and read
// with the transposing LDS load of gfx950 (ds_read_b64_tr_b16), which hands each
// lane four consecutive contraction elements of one operand row.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int BK = 64;
constexpr int ROW_BYTES = BK * 2;  // 128

struct GemmDev {
    const bf16_t* A; const bf16_t* W; void* C; const float* R; const bf16_t* bias;
    int lda, ldw, ldc, ldr;
    int M, N, K;
    int tilesM, tilesN;
};

__device__ __forceinline__ int lds_off(int row, int chunk) {
    return row * ROW_BYTES + ((chunk ^ ((row >> 1) & 7)) << 4);
}

// ---- tile loaders -----------------------------------------------------------
// K-major source: rows of 64 contiguous k. ROWS*8 16-byte chunks over 256 threads.
template <int ROWS, int NT>
struct LoaderK {
    static constexpr int ITERS = ROWS * 8 / NT;
    static constexpr int N_LOADS = ITERS, N_STORES = ITERS;   // per thread and tile
    const bf16_t* src[ITERS];
    int dst[ITERS];
    u32x4_t regs[ITERS];
    // row_of(r) maps a tile row to a (clamped) global row.
    template <class RowMap>
    __device__ __forceinline__ void init(const bf16_t* base, int ld, RowMap row_of) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int q = threadIdx.x + i * NT;
            const int row = q >> 3, c = q & 7;
            src[i] = base + (size_t)row_of(row) * ld + c * 8;
            dst[i] = lds_off(row, c);
        }
    }
    __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) regs[i] = *reinterpret_cast<const u32x4_t*>(src[i] + k0);
    }
    __device__ __forceinline__ void store(unsigned char* lds) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) *reinterpret_cast<u32x4_t*>(lds + dst[i]) = regs[i];
    }
};

// Row-major source (element (r,k) at base[k*ld + r]): the tile is copied as it lies in
// memory -- LDS row = contraction index k (64 rows), ROWS contiguous r values per row, rows
// padded by 64 bytes -- with the same coalesced 16-byte chunks as above.  The transposition
// happens in the fragment read (ds_read_b64_tr_b16, see tr_frag below).
template <int ROWS>
struct TLayout {
    static constexpr int STRIDE = ROWS * 2 + 64;   // bytes per k row
    static constexpr int BYTES = BK * STRIDE;
};

template <int ROWS, int NT>
struct LoaderR {
    static constexpr int CPR = ROWS / 8;           // 16-byte chunks per k row
    static constexpr int ITERS = BK * CPR / NT;
    static constexpr int N_LOADS = ITERS, N_STORES = ITERS;
    const bf16_t* src[ITERS];
    int dst[ITERS];
    int ld_;
    u32x4_t regs[ITERS];
    // col_of(r) maps the tile's first r of a chunk to a (clamped) global r.
    template <class ColMap>
    __device__ __forceinline__ void init(const bf16_t* base, int ld, ColMap col_of) {
        ld_ = ld;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int q = threadIdx.x + i * NT;
            const int k = q / CPR, c = q % CPR;
            src[i] = base + (size_t)k * ld + col_of(c * 8);
            dst[i] = k * TLayout<ROWS>::STRIDE + c * 16;
        }
    }
    __device__ __forceinline__ void fetch(int k0) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) regs[i] = *reinterpret_cast<const u32x4_t*>(src[i] + (size_t)k0 * ld_);
    }
    __device__ __forceinline__ void store(unsigned char* lds) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) *reinterpret_cast<u32x4_t*>(lds + dst[i]) = regs[i];
    }
};

// Fragment of a 32-row MFMA operand out of a k-row tile.  ds_read_b64_tr_b16 works on
// groups of 16 lanes: lane s of a group supplies the address of an 8-byte block (4 values of
// one k row), and lane i receives element i%4 of the blocks supplied by lanes i/4, i/4+4,
// i/4+8, i/4+12 (layout checked on the device with an index pattern).  With lane s pointing at
// k row (s>>2) and r block 4*(s&3), lane i ends up with r = 4*(i>>2) + (i&3) = i and four
// consecutive k: two reads give the eight k of a lane's operand, in the same order as the
// 16-byte read of a k-contiguous tile, so both operand forms can be mixed.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

__device__ __forceinline__ bf16x8_t tr_frag(const unsigned char* p, int stride) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * stride));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, both);
}

template <int ROWS, int NT, int FORM>
struct LoaderSel { typedef LoaderK<ROWS, NT> type; };
template <int ROWS, int NT>
struct LoaderSel<ROWS, NT, OP_RMAJOR> { typedef LoaderR<ROWS, NT> type; };

// Epilogue shared by the GEMM kernels.  acc[j][i] is the 32x32 tile (n tile j, m tile i) of
// a wave whose first row is m_base and first output column n_base; a lane holds row l32 of
// the m tile and, in register e, column j*32 + (e/4)*8 + half*4 + e%4.
template <int EPI, int TM, int TN>
__device__ __forceinline__ void gemm_epilogue(const GemmDev& p, f32x16_t (&acc)[TN][TM], int m_base, int n_base,
                                              int l32, int half) {
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU_BF16);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m_base + i * 32 + l32;
        if (m >= p.M) continue;
        if (SWIGLU) {
#pragma unroll
            for (int j = 0; j < TN / 2; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n_base + j * 32 + g * 8 + half * 4;
                    if (n >= p.N) continue;
                    float z[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gv = acc[j][i][g * 4 + e], uv = acc[j + TN / 2][i][g * 4 + e];
                        z[e] = gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * uv;
                    }
                    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(p.C) + (size_t)m * p.ldc + n) =
                        make_uint2(pack_bf2(z[0], z[1]), pack_bf2(z[2], z[3]));
                }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n_base + j * 32 + g * 8 + half * 4;
                    if (n >= p.N) continue;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[j][i][g * 4 + e];
                    if (p.bias) {
                        const uint2 b = *reinterpret_cast<const uint2*>(p.bias + n);
                        v[0] += bf_lo(b.x); v[1] += bf_hi(b.x); v[2] += bf_lo(b.y); v[3] += bf_hi(b.y);
                    }
                    if (EPI == EPI_RESID_F32) {
                        const float4 r = *reinterpret_cast<const float4*>(p.R + (size_t)m * p.ldr + n);
                        *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.C) + (size_t)m * p.ldc + n) =
                            make_float4(r.x + v[0], r.y + v[1], r.z + v[2], r.w + v[3]);
                    } else if (EPI == EPI_F32) {
                        *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.C) + (size_t)m * p.ldc + n) =
                            make_float4(v[0], v[1], v[2], v[3]);
                    } else {
                        if (EPI == EPI_GELU_BF16) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
                        }
                        *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(p.C) + (size_t)m * p.ldc + n) =
                            make_uint2(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]));
                    }
                }
        }
    }
}


// ---- the kernel ---------------------------------------------------------------
template <int BM, int BN, int EPI, int AFORM, int WFORM, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_kernel(GemmDev p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int NT = WAVES * 64;
    constexpr int WNC = WAVES / 2;               // wave grid: 2 (m) x WNC (n)
    constexpr int WN = BN / WNC;                 // tile rows of W per wave column
    constexpr int TM = BM / 64, TN = WN / 32;    // 32x32 tiles per wave
    constexpr int A_BYTES = AFORM == OP_KMAJOR ? BM * ROW_BYTES : TLayout<BM>::BYTES;
    constexpr int W_BYTES = WFORM == OP_KMAJOR ? BN * ROW_BYTES : TLayout<BN>::BYTES;
    constexpr int STAGE = A_BYTES + W_BYTES;
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU_BF16);
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;  // output columns per block
    static_assert(!SWIGLU || (TN % 2 == 0), "gate and up tiles pair up inside a wave");

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, half = lane >> 5;

    // XCD-aware, grouped tile order: 8 m-tiles share each n-tile back to back.
    int pid = xcd_remap(blockIdx.x, gridDim.x);
    constexpr int GM = 8;
    const int group = GM * p.tilesN;
    const int first_m = (pid / group) * GM;
    const int gm = min(p.tilesM - first_m, GM);
    const int tm = first_m + (pid % group) % gm;
    const int tn = (pid % group) / gm;
    const int m0 = tm * BM, n0 = tn * BN_OUT;

    typename LoaderSel<BM, NT, AFORM>::type la;
    typename LoaderSel<BN, NT, WFORM>::type lw;
    {
        const int M = p.M, N = p.N;
        if (AFORM == OP_KMAJOR)
            la.init(p.A, p.lda, [=](int r) { return min(m0 + r, M - 1); });
        else
            la.init(p.A, p.lda, [=](int r) { return min(m0 + r, M - 8); });
        if (SWIGLU) {
            // tile row r -> wave column wr, 32-row tile j; first half of a wave's
            // tiles are gate rows, second half the matching up rows (offset N).
            lw.init(p.W, p.ldw, [=](int r) {
                const int wr = r / WN, j = (r % WN) >> 5, rr = r & 31;
                const int isup = j >= TN / 2;
                const int col = n0 + wr * (WN / 2) + (isup ? j - TN / 2 : j) * 32 + rr;
                return min(col, N - 1) + (isup ? N : 0);
            });
        } else if (WFORM == OP_KMAJOR) {
            lw.init(p.W, p.ldw, [=](int r) { return min(n0 + r, N - 1); });
        } else {
            lw.init(p.W, p.ldw, [=](int r) { return min(n0 + r, N - 8); });
        }
    }

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

    // per-lane fragment offsets: row l32 of a 32-row tile, chunk 2*ks + half
    const int sw = (l32 >> 1) & 7;
    int foff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) foff[ks] = l32 * ROW_BYTES + (((2 * ks + half) ^ sw) << 4);
    // k-row tiles: lane -> k row 8*half + (s>>2), r block 16*((lane>>4)&1) + 4*(s&3), s = lane&15
    const int s16 = lane & 15;
    const int tro_a = (8 * half + (s16 >> 2)) * TLayout<BM>::STRIDE + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
    const int tro_w = (8 * half + (s16 >> 2)) * TLayout<BN>::STRIDE + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
    const int a_base = AFORM == OP_KMAJOR ? wm * (BM / 2) * ROW_BYTES : wm * (BM / 2) * 2 + tro_a;
    const int w_base = A_BYTES + (WFORM == OP_KMAJOR ? wn * WN * ROW_BYTES : wn * WN * 2 + tro_w);

    const int KT = p.K / BK;
    la.fetch(0);
    lw.fetch(0);
    la.store(smem);
    lw.store(smem + A_BYTES);
    __syncthreads();

    // Main loop, one barrier per 64-deep tile.  The body is branch-free (the last
    // iteration re-fetches the last tile into the idle buffer) so that it is one
    // scheduling region; fragments are double buffered in registers and the
    // scheduling hints interleave the LDS reads of step s+1 with the MFMAs of step
    // s, and the LDS stores of the next tile with the MFMAs of the last step.
    constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
    typedef typename LoaderSel<BM, NT, AFORM>::type LA;
    typedef typename LoaderSel<BN, NT, WFORM>::type LW;
    constexpr int LA_LOADS = LA::N_LOADS, LW_LOADS = LW::N_LOADS, LA_STORES = LA::N_STORES, LW_STORES = LW::N_STORES;
    constexpr int M_MFMA = 0x008, M_VMEM_RD = 0x020, M_DS_RD = 0x100, M_DS_WR = 0x200;
    for (int kt = 0; kt < KT; ++kt) {
        unsigned char* cur = smem + (kt & 1) * STAGE;
        unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
        const int knext = min(kt + 1, KT - 1) * BK;
        bf16x8_t af[2][TM], wf[2][TN];
        auto load_frags = [&](int ks, int buf) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[buf][i] = AFORM == OP_KMAJOR
                                 ? *reinterpret_cast<const bf16x8_t*>(cur + a_base + i * 32 * ROW_BYTES + foff[ks])
                                 : tr_frag(cur + a_base + i * 64 + ks * 16 * TLayout<BM>::STRIDE, TLayout<BM>::STRIDE);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                wf[buf][j] = WFORM == OP_KMAJOR
                                 ? *reinterpret_cast<const bf16x8_t*>(cur + w_base + j * 32 * ROW_BYTES + foff[ks])
                                 : tr_frag(cur + w_base + j * 64 + ks * 16 * TLayout<BN>::STRIDE, TLayout<BN>::STRIDE);
        };
        load_frags(0, 0);
        la.fetch(knext);
        lw.fetch(knext);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) {
                load_frags(ks + 1, (ks + 1) & 1);
            } else {
                la.store(nxt);
                lw.store(nxt + A_BYTES);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][j], af[ks & 1][i], acc[j][i], 0, 0, 0);
        }
        // One pipeline description for the whole body, in issue order: the step-0
        // fragments; then per step 2 MFMAs per fragment read of the next step (the
        // tile's global loads ride along in step 0); in the last step one LDS store
        // of the next tile per MFMA.
        constexpr int AR = AFORM == OP_KMAJOR ? 1 : 2, WR = WFORM == OP_KMAJOR ? 1 : 2;   // LDS reads per fragment
        __builtin_amdgcn_sched_group_barrier(M_DS_RD, TM * AR + TN * WR, 0);
#pragma unroll
        for (int ks = 0; ks < 3; ++ks) {
#pragma unroll
            for (int i = 0; i < NFRAG; ++i) {
                __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA / NFRAG, 0);
                if (i < TM) __builtin_amdgcn_sched_group_barrier(M_DS_RD, AR, 0);
                else __builtin_amdgcn_sched_group_barrier(M_DS_RD, WR, 0);
                if (ks == 0) __builtin_amdgcn_sched_group_barrier(M_VMEM_RD, (LA_LOADS + LW_LOADS + NFRAG - 1) / NFRAG, 0);
            }
            if (NMFMA % NFRAG) __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA % NFRAG, 0);
        }
#pragma unroll
        for (int i = 0; i < NMFMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(M_MFMA, 1, 0);
            __builtin_amdgcn_sched_group_barrier(M_DS_WR, (LA_STORES + LW_STORES + NMFMA - 1) / NMFMA, 0);
        }
        __syncthreads();
    }

    gemm_epilogue<EPI, TM, TN>(p, acc, m0 + wm * (BM / 2), SWIGLU ? n0 + wn * (WN / 2) : n0 + wn * WN, l32, half);
}

// Epilogue through LDS (used by the LDS-DMA kernel, whose LDS is idle once the k-loop ends).
// Written straight from the accumulators a store instruction covers 32 rows x 16 or 32 bytes:
// 2 M write requests of 16 bytes per round of 256 tiles, which the L2 takes ~9 us to absorb
// (a fifth of the ViT-H first MLP projection).  Here the values (bias, GELU, SwiGLU applied)
// are first laid out in LDS as the output tile, RP rows at a time (row stride + 16 bytes: a
// wave's 32 rows spread over the banks), and then written with 16 bytes per lane, consecutive
// lanes on consecutive bytes of a row: whole 128-byte lines.  The residual is read the same way.
// acc[j][i]: tile (n tile j, m tile i) of a wave whose first tile row is wrow0 and first output
// column inside the tile wcol0; lane layout as in gemm_epilogue.
template <int EPI, int TM, int TN, int BM, int BN_OUT, int NT, int LDS_BYTES>
__device__ __forceinline__ void gemm_epilogue_staged(const GemmDev& p, f32x16_t (&acc)[TN][TM], unsigned char* smem,
                                                     int m0, int n0, int wrow0, int wcol0, int l32, int half) {
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU_BF16);
    constexpr bool F32OUT = (EPI == EPI_RESID_F32 || EPI == EPI_F32);
    constexpr int ESZ = F32OUT ? 4 : 2;
    constexpr int ROWB = BN_OUT * ESZ, STRIDE = ROWB + 16;
    constexpr int BIAS_BYTES = BN_OUT * 2;                // the tile's bias values, staged behind the passes
    constexpr int ROOM = LDS_BYTES - BIAS_BYTES;
    constexpr int RP = BM * STRIDE <= ROOM ? BM : (BM / 2) * STRIDE <= ROOM ? BM / 2 : BM / 4;
    static_assert(RP * STRIDE <= ROOM && RP % 32 == 0 && BIAS_BYTES % 16 == 0, "a pass of the output tile fits the LDS");
    const bf16_t* sbias = reinterpret_cast<const bf16_t*>(smem + ROOM);
    constexpr int TNO = SWIGLU ? TN / 2 : TN;
    constexpr int CPR = ROWB / 16, CHUNKS = RP * CPR;     // 16-byte chunks per row / per pass
    // the values of 4 consecutive columns (register group g of tile (j, i))
    auto values = [&](int i, int j, int g, float (&v)[4]) {
        const int nl = wcol0 + j * 32 + g * 8 + half * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (SWIGLU) {
                const float gv = acc[j][i][g * 4 + e], uv = acc[j + TN / 2][i][g * 4 + e];
                v[e] = gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * uv;
            } else {
                v[e] = acc[j][i][g * 4 + e];
            }
        }
        if (!SWIGLU && p.bias) {
            const uint2 b = *reinterpret_cast<const uint2*>(sbias + nl);
            v[0] += bf_lo(b.x); v[1] += bf_hi(b.x); v[2] += bf_lo(b.y); v[3] += bf_hi(b.y);
        }
        if (EPI == EPI_GELU_BF16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
        }
    };
    __syncthreads();   // every wave is done with the operand stages, no load is in flight
    // Barriers from here on order LDS traffic only (lgkmcnt): a __syncthreads() would also wait
    // for the global stores of a pass to be acknowledged, several microseconds per pass with the
    // matrix pipes idle.
    constexpr int WAIT_LGKM0 = 15 | (7 << 4) | (0 << 8) | (3 << 14);   // vmcnt 63, expcnt 7, lgkmcnt 0
    auto lds_barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // The tile's bias values go through LDS once: fetched from global memory where they are used,
    // every one of a lane's TM x TN x 4 little loads was waited for in turn (a cache round trip each).
    if (!SWIGLU && p.bias) {
        for (int c = threadIdx.x; c < BN_OUT / 8; c += NT) {
            const int n = n0 + c * 8;
            const u32x4_t b = n < p.N ? *reinterpret_cast<const u32x4_t*>(p.bias + n) : u32x4_t{0, 0, 0, 0};   // N % 8 == 0
            *reinterpret_cast<u32x4_t*>(smem + ROOM + c * 16) = b;
        }
        lds_barrier();
    }
    // bf16 outputs: every wave computes and packs all of its values first (the activation
    // functions are the expensive part and must not be serialised by the passes below)
    uint2 pk[F32OUT ? 1 : TM][F32OUT ? 1 : TNO][4];
    if (!F32OUT) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TNO; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v[4];
                    values(i, j, g, v);
                    pk[F32OUT ? 0 : i][F32OUT ? 0 : j][g] = make_uint2(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]));
                }
    }
    // A thread's residual loads of a pass are all issued before the first is used (one after the
    // other, each waited for, they cost a memory round trip per 16 bytes), the first batch before
    // the pass's LDS writes, so that its latency runs under those.
    constexpr int ITER = (CHUNKS + NT - 1) / NT;
    constexpr int SB = ITER > 6 ? (ITER + 1) / 2 : ITER;     // residual pieces in flight per thread
    auto chunk_pos = [&](int pass, int it, int* row, int* ch, int* m, int* n) {
        const int c = threadIdx.x + it * NT;
        *row = c / CPR;
        *ch = c % CPR;
        *m = m0 + pass * RP + *row;
        *n = n0 + *ch * (16 / ESZ);
        return c < CHUNKS && *m < p.M && *n < p.N;
    };
    float4 rr[EPI == EPI_RESID_F32 ? SB : 1];
    auto load_resid = [&](int pass, int it0) {
#pragma unroll
        for (int it = it0; it < it0 + SB && it < ITER; ++it) {
            int row, ch, m, n;
            const bool ok = chunk_pos(pass, it, &row, &ch, &m, &n);
            rr[it - it0] = ok ? *reinterpret_cast<const float4*>(p.R + (size_t)m * p.ldr + n) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
#pragma unroll
    for (int pass = 0; pass < BM / RP; ++pass) {
        if (EPI == EPI_RESID_F32) load_resid(pass, 0);
        if (pass) lds_barrier();     // the previous pass has been read out
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wrow0 + i * 32;                 // wave-uniform
            if (r / RP != pass) continue;
            unsigned char* rowp = smem + (r - pass * RP + l32) * STRIDE;
#pragma unroll
            for (int j = 0; j < TNO; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int nl = wcol0 + j * 32 + g * 8 + half * 4;
                    if (F32OUT) {
                        float v[4];
                        values(i, j, g, v);
                        *reinterpret_cast<float4*>(rowp + nl * 4) = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
                        *reinterpret_cast<uint2*>(rowp + nl * 2) = pk[F32OUT ? 0 : i][F32OUT ? 0 : j][g];
                    }
                }
        }
        lds_barrier();
#pragma unroll
        for (int it0 = 0; it0 < ITER; it0 += SB) {
            if (EPI == EPI_RESID_F32 && it0) load_resid(pass, it0);
#pragma unroll
            for (int it = it0; it < it0 + SB && it < ITER; ++it) {
                int row, ch, m, n;
                if (chunk_pos(pass, it, &row, &ch, &m, &n)) {
                    u32x4_t v = *reinterpret_cast<const u32x4_t*>(smem + row * STRIDE + ch * 16);
                    if (EPI == EPI_RESID_F32) {
                        const float4 a = __builtin_bit_cast(float4, v);
                        const float4 r = rr[it - it0];
                        v = __builtin_bit_cast(u32x4_t, make_float4(a.x + r.x, a.y + r.y, a.z + r.z, a.w + r.w));
                    }
                    *reinterpret_cast<u32x4_t*>(static_cast<unsigned char*>(p.C) + ((size_t)m * p.ldc + n) * ESZ) = v;
                }
            }
        }
    }
}

// ---- LDS-DMA kernel (both operands contraction-contiguous) ----------------------------------
// Global loads write LDS directly (global_load_lds_dwordx4): no staging registers and no
// ds_write instructions.  Measured on MI355X, LDS writes issued by the waves run at about
// 75 bytes/clk per CU and serialise with the fragment reads (215 bytes/clk), so a 256x256x64
// tile costs ~870 + ~900 LDS cycles against 2048 MFMA cycles; the DMA writes overlap the reads.
// A wave instruction lands 64 lanes x 16 bytes = 8 tile rows of 128 bytes contiguously, so the
// XOR swizzle of the 16-byte chunks is applied on the global side (which chunk a lane fetches);
// the LDS image is the one the register-staged kernel builds.
//
// Two 64-deep stages.  The only barrier of a tile sits before its LAST k-step: by then a wave
// has read all its fragments of the tile (the last step's are in registers) and its loads of the
// next tile, issued one tile earlier, have landed, so after the barrier the other stage is
// readable and this stage is free.  The last step then runs with the first fragments of the
// next tile being read under its MFMAs: nothing that follows the barrier waits on memory.
// The loads of a tile are spread over three k-steps (after the barrier, then steps 0 and 1 of
// the next tile): issued in one burst they fill the address unit's queue and stall the
// wave's MFMAs behind them (253 -> 231 us on the gate/up shape with zero operands).
// The compiler does not order these loads against later LDS reads; the kernel waits with
// explicit vmcnt/lgkmcnt counts and uses a bare s_barrier (the fence of __syncthreads() is
// what the counts replace).
typedef __attribute__((address_space(3))) void* lds_void_ptr;

template <int BM, int BN, int EPI, int WAVES, int WM>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 2 : 1) void gemm_dma_kernel(GemmDev p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int WNC = WAVES / WM;              // wave grid: WM (m) x WNC (n)
    constexpr int WMR = BM / WM, WN = BN / WNC;  // tile rows of A / of W per wave
    constexpr int TM = WMR / 32, TN = WN / 32;   // 32x32 tiles per wave
    static_assert(WMR % 32 == 0 && WN % 32 == 0, "whole MFMA tiles per wave");
    constexpr int A_BYTES = BM * ROW_BYTES, STAGE = (BM + BN) * ROW_BYTES;
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU_BF16);
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    constexpr int NBLK_A = BM / 8, NBLK = (BM + BN) / 8;   // 1 KiB load blocks (8 tile rows each)
    constexpr int NI = NBLK / WAVES;           // load instructions per wave and stage
    constexpr int N_AFTER = (3 * NI + 7) / 8;  // of those: issued right after the barrier,
    constexpr int N_STEP0 = N_AFTER < NI - N_AFTER ? N_AFTER : NI - N_AFTER;   // in step 0 (rest: step 1)
    static_assert(NBLK % WAVES == 0, "whole load blocks per wave");
    static_assert(!SWIGLU || (TN % 2 == 0), "gate and up tiles pair up inside a wave");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int l32 = lane & 31, half = lane >> 5;

    int pid = xcd_remap(blockIdx.x, gridDim.x);
    constexpr int GM = 8;
    const int group = GM * p.tilesN;
    const int first_m = (pid / group) * GM;
    const int gm = min(p.tilesM - first_m, GM);
    const int tm = first_m + (pid % group) % gm;
    const int tn = (pid % group) / gm;
    const int m0 = tm * BM, n0 = tn * BN_OUT;

    // load assignment: block b of 8 tile rows, b < BM/8 -> A rows, else W rows.  Lane l lands at
    // row l>>3, 16-byte position l&7 of the block, and fetches the chunk that the swizzle puts there.
    const bf16_t* src[NI];
    int dst[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int blk = wave * NI + i;
        const bool is_w = blk >= NBLK_A;
        const int row = (is_w ? blk - NBLK_A : blk) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        if (is_w) {
            int grow;
            if (SWIGLU) {
                const int wr = row / WN, j = (row % WN) >> 5, rr = row & 31;
                const int isup = j >= TN / 2;
                const int col = n0 + wr * (WN / 2) + (isup ? j - TN / 2 : j) * 32 + rr;
                grow = min(col, p.N - 1) + (isup ? p.N : 0);
            } else {
                grow = min(n0 + row, p.N - 1);
            }
            src[i] = p.W + (size_t)grow * p.ldw + chunk * 8;
        } else {
            src[i] = p.A + (size_t)min(m0 + row, p.M - 1) * p.lda + chunk * 8;
        }
        dst[i] = blk * 8 * ROW_BYTES;
    }
    const int KT = p.K / BK;
    // (The builtin's address-space-qualified parameters do not type-check in the host pass
    // of a template, which would silently drop the kernel's host stub: device pass only.)
#if defined(__HIP_DEVICE_COMPILE__)
#define SP_DMA_ISSUE(tile, stage) SP_DMA_ISSUE_R(tile, stage, 0, NI)
#define SP_DMA_ISSUE_R(tile, stage, i0, i1)                                                                   \
    do {                                                                                                       \
        const int k0_ = min((tile), KT - 1) * BK;                                                              \
        _Pragma("unroll") for (int i_ = (i0); i_ < (i1); ++i_)                                                 \
            __builtin_amdgcn_global_load_lds(src[i_] + k0_, (lds_void_ptr)(smem + (stage) * STAGE + dst[i_]), \
                                             16, 0, 0);                                                        \
    } while (0)
#else
#define SP_DMA_ISSUE(tile, stage) ((void)src, (void)dst)
#define SP_DMA_ISSUE_R(tile, stage, i0, i1) ((void)src, (void)dst)
#endif

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

    const int sw = (l32 >> 1) & 7;
    int foff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) foff[ks] = l32 * ROW_BYTES + (((2 * ks + half) ^ sw) << 4);
    const int a_base = wm * WMR * ROW_BYTES;
    const int w_base = A_BYTES + wn * WN * ROW_BYTES;

    constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
    constexpr int M_MFMA = 0x008, M_VMEM_RD = 0x020, M_DS_RD = 0x100;
    // s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
    constexpr int WAIT_VM0_LGKM0 = (0 & 15) | (7 << 4) | (0 << 8) | (0 << 14);
    constexpr int WAIT_VM_AFTER = (N_AFTER & 15) | (7 << 4) | (15 << 8) | ((N_AFTER >> 4) << 14);

    bf16x8_t af[2][TM], wf[2][TN];
    auto load_frags = [&](const unsigned char* tile, int ks, int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[buf][i] = *reinterpret_cast<const bf16x8_t*>(tile + a_base + i * 32 * ROW_BYTES + foff[ks]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            wf[buf][j] = *reinterpret_cast<const bf16x8_t*>(tile + w_base + j * 32 * ROW_BYTES + foff[ks]);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][j], af[buf][i], acc[j][i], 0, 0, 0);
    };

    SP_DMA_ISSUE(0, 0);
    SP_DMA_ISSUE_R(1, 1, 0, N_AFTER);
    __builtin_amdgcn_s_waitcnt(WAIT_VM_AFTER);      // this thread's loads of tile 0 have landed
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    load_frags(smem, 0, 0);
    for (int kt = 0; kt < KT; ++kt) {
        unsigned char* cur = smem + (kt & 1) * STAGE;
        unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
        // the rest of tile kt+1's loads (its first N_AFTER went out after the last barrier)
        SP_DMA_ISSUE_R(kt + 1, (kt + 1) & 1, N_AFTER, N_AFTER + N_STEP0);
        load_frags(cur, 1, 1);
        mfmas(0);
        SP_DMA_ISSUE_R(kt + 1, (kt + 1) & 1, N_AFTER + N_STEP0, NI);
        load_frags(cur, 2, 0);
        mfmas(1);
        load_frags(cur, 3, 1);
        mfmas(0);
#define SP_SCHED_STEP(NV)                                                                  \
        _Pragma("unroll") for (int i = 0; i < NFRAG; ++i) {                                    \
            __builtin_amdgcn_sched_group_barrier(M_DS_RD, 1, 0);                               \
            __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA / NFRAG, 0);                    \
            if (i < (NV)) __builtin_amdgcn_sched_group_barrier(M_VMEM_RD, 1, 0);                  \
        }                                                                                      \
        if (NMFMA % NFRAG) __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA % NFRAG, 0);
        SP_SCHED_STEP(N_STEP0)
        SP_SCHED_STEP(NI - N_AFTER - N_STEP0)
        SP_SCHED_STEP(0)
#undef SP_SCHED_STEP
        // This wave's reads of tile kt are complete and its loads of tile kt+1 (issued one tile
        // ago) have landed; after the barrier that holds for every wave, so the other stage is
        // readable and this stage may be refilled.
        __builtin_amdgcn_s_waitcnt(WAIT_VM0_LGKM0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        SP_DMA_ISSUE_R(kt + 2, kt & 1, 0, N_AFTER);
        load_frags(nxt, 0, 0);
        mfmas(1);
#pragma unroll
        for (int i = 0; i < NFRAG; ++i) {
            __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA / NFRAG, 0);
            __builtin_amdgcn_sched_group_barrier(M_DS_RD, 1, 0);
        }
        if (NMFMA % NFRAG) __builtin_amdgcn_sched_group_barrier(M_MFMA, NMFMA % NFRAG, 0);
    }
    __builtin_amdgcn_s_waitcnt(WAIT_VM0_LGKM0);   // drain the tail's idle loads
    gemm_epilogue_staged<EPI, TM, TN, BM, BN_OUT, WAVES * 64, 2 * STAGE>(p, acc, smem, m0, n0, wm * WMR,
                                                                         SWIGLU ? wn * (WN / 2) : wn * WN, l32, half);
#undef SP_DMA_ISSUE
#undef SP_DMA_ISSUE_R
}

template <int BM, int BN, int EPI, int WAVES, int WM>
hipError_t launch_dma(hipStream_t st, const GemmArgs& g) {
    constexpr int LDS = 2 * (BM + BN) * ROW_BYTES;
    constexpr int BN_OUT = (EPI == EPI_SWIGLU_BF16) ? BN / 2 : BN;
    static LdsLimitOnce lds_limit;
    hipError_t e = lds_limit.set(reinterpret_cast<const void*>(gemm_dma_kernel<BM, BN, EPI, WAVES, WM>), LDS);
    if (e != hipSuccess) return e;
    GemmDev d;
    d.A = g.A; d.W = g.W; d.C = g.C; d.R = g.R; d.bias = g.bias;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc; d.ldr = g.ldr;
    d.M = g.M; d.N = g.N; d.K = g.K;
    d.tilesM = (g.M + BM - 1) / BM;
    d.tilesN = (g.N + BN_OUT - 1) / BN_OUT;
    gemm_dma_kernel<BM, BN, EPI, WAVES, WM><<<d.tilesM * d.tilesN, WAVES * 64, LDS, st>>>(d);
    return hipGetLastError();
}

template <int BM, int BN, int EPI, int AFORM, int WFORM, int WAVES>
hipError_t launch_one(hipStream_t st, const GemmArgs& g) {
    constexpr int LDS = 2 * ((AFORM == OP_KMAJOR ? BM * ROW_BYTES : TLayout<BM>::BYTES) +
                             (WFORM == OP_KMAJOR ? BN * ROW_BYTES : TLayout<BN>::BYTES));
    constexpr int BN_OUT = (EPI == EPI_SWIGLU_BF16) ? BN / 2 : BN;
    static LdsLimitOnce lds_limit;   // one per instantiation
    auto kern = gemm_kernel<BM, BN, EPI, AFORM, WFORM, WAVES>;
    hipError_t e = lds_limit.set(reinterpret_cast<const void*>(kern), LDS);
    if (e != hipSuccess) return e;
    GemmDev d;
    d.A = g.A; d.W = g.W; d.C = g.C; d.R = g.R; d.bias = g.bias;
    d.lda = g.lda; d.ldw = g.ldw; d.ldc = g.ldc; d.ldr = g.ldr;
    d.M = g.M; d.N = g.N; d.K = g.K;
    d.tilesM = (g.M + BM - 1) / BM;
    d.tilesN = (g.N + BN_OUT - 1) / BN_OUT;
    const int nblocks = d.tilesM * d.tilesN;
    gemm_kernel<BM, BN, EPI, AFORM, WFORM, WAVES><<<nblocks, WAVES * 64, LDS, st>>>(d);
    return hipGetLastError();
}

// Tile ids: register-staged kernel 1 = 128x128, 2 = 128x256 (BM x BN), 3 = 256x256 (4 waves each),
// 4 = 256x256 with 8 waves; LDS-DMA kernel (contraction-contiguous operands only) 5 = 256x256 and
// 6 = 128x256 with 8 waves, 7 = 128x128 with 4 waves (two work-groups per CU), 8 = 256x192 with 8
// waves in a 4 x 2 grid (not with the SwiGLU epilogue, which pairs tiles inside a wave); 9 = the
// weight-streaming kernel for at most 64 activation rows (k_gemm_skinny.hip); 10 = 256x320 of the
// LDS-DMA kernel, 4 x 2 waves (not with SwiGLU): N = 1280 is four of its columns, so the ViT-H
// projections back to d_model are one round of 256 work-groups once the ragged rows are cut off.
//
// Choice (shapes only, so a stack's kernels never depend on the streaming window): the chip
// runs 256 work-groups at a time (512 of tile 7), so a launch costs
// ceil(tiles / concurrent) rounds of one tile's time; a tile's time is its area over a measured
// relative efficiency (larger tiles move fewer operand bytes per MFMA).  Take the cheapest.
// (Activation rows are contiguous in A, C and R, so a launch can be cut along M.)
struct TileCost { int id, bm, bn, concurrent; float eff; };
constexpr TileCost kDmaTiles[] = {{5, 256, 256, 256, 1.00f}, {10, 256, 320, 256, 1.02f}, {8, 256, 192, 256, 0.85f},
                                  {6, 128, 256, 256, 0.72f}, {7, 128, 128, 512, 0.70f}};
constexpr TileCost kRegTiles[] = {{4, 256, 256, 256, 1.00f}, {1, 128, 128, 512, 0.66f}};

template <int NC>
int pick_tile(const TileCost (&cand)[NC], int M, int N, int epi, float* cost_out = nullptr) {
    int best = cand[0].id;
    float best_cost = 0.f;
    for (int c = 0; c < NC; ++c) {
        const TileCost& t = cand[c];
        if ((t.id == 8 || t.id == 10) && epi == EPI_SWIGLU_BF16) continue;
        const int bn_out = (epi == EPI_SWIGLU_BF16) ? t.bn / 2 : t.bn;
        const long tiles = (long)((M + t.bm - 1) / t.bm) * ((N + bn_out - 1) / bn_out);
        // in units of "every CU busy with one tile": the two-per-CU tile fills a CU with two
        long units = tiles / t.concurrent * (t.concurrent / 256);
        const long rem = tiles % t.concurrent;
        if (rem) units += rem <= 256 ? 1 : t.concurrent / 256;
        const float cost = (float)units * (float)(t.bm * t.bn) / t.eff;
        if (c == 0 || cost < best_cost) { best = t.id; best_cost = cost; }   // candidate 0 takes every epilogue
    }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// The library's own choice for a shape: the tile, and when a ragged last row of 256-row tiles
// would cost a whole extra round (ViT-H: 16448 tokens = 64 tiles + 64 rows, 1300 tiles = 5.08
// rounds of 256) the rows beyond the last multiple of 256 become a launch of their own.
GemmPlan plan_gemm(int epi, bool dma_ok, int M, int N) {
    GemmPlan pl{0, M, 0};
    if (!dma_ok) {
        pl.tile = pick_tile(kRegTiles, M, N, epi);
        return pl;
    }
    if (M <= SPK_SKINNY_MAX_ROWS) {     // a decode step: nothing of W is re-used, stream it
        pl.tile = 9;
        return pl;
    }
    float whole;
    pl.tile = pick_tile(kDmaTiles, M, N, epi, &whole);
    const int tail = M % 256, body = M - tail;
    if (tail && body) {
        float c_body, c_tail;
        const int t_body = pick_tile(kDmaTiles, body, N, epi, &c_body);
        int t_tail;
        if (tail <= SPK_SKINNY_MAX_ROWS) {
            // the weight-streaming kernel in the units of pick_tile (a round of 256x256 tiles = 65536):
            // N x K x 2 bytes at ~4.5 TB/s against 256 tiles x 2 x 65536 K flop at ~1.3 PFLOP/s, plus a launch
            t_tail = 9;
            c_tail = 1.13f * (float)N + 6000.f;
        } else {
            t_tail = pick_tile(kDmaTiles, tail, N, epi, &c_tail);
        }
        if (c_body + c_tail < 0.97f * whole) pl = GemmPlan{t_body, body, t_tail};
    }
    return pl;
}

template <int EPI, int AFORM, int WFORM>
hipError_t launch_tile(hipStream_t st, const GemmArgs& g) {
    constexpr bool DMA_OK = (AFORM == OP_KMAJOR && WFORM == OP_KMAJOR);
    constexpr int NOSWIGLU = EPI == EPI_SWIGLU_BF16 ? EPI_BF16 : EPI;   // tile 8 has an odd tile count per wave
    constexpr size_t CSZ = (EPI == EPI_RESID_F32 || EPI == EPI_F32) ? 4 : 2;
    // the LDS-DMA kernel writes C (and reads R) in 16-byte pieces of a row
    const bool dma = DMA_OK && (g.ldc * CSZ) % 16 == 0;
    int tile = g.tile;
    if (!tile) {
        const GemmPlan pl = plan_gemm(EPI, dma, g.M, g.N);
        tile = pl.tile;
        if (pl.body_rows < g.M) {
            GemmArgs a = g, b = g;
            a.M = pl.body_rows; a.tile = pl.tile;
            b.M = g.M - pl.body_rows; b.tile = pl.tail_tile;
            b.A = g.A + (size_t)pl.body_rows * g.lda;
            b.C = static_cast<unsigned char*>(g.C) + (size_t)pl.body_rows * g.ldc * CSZ;
            if (g.R) b.R = g.R + (size_t)pl.body_rows * g.ldr;
            hipError_t e = launch_tile<EPI, AFORM, WFORM>(st, a);
            return e != hipSuccess ? e : launch_tile<EPI, AFORM, WFORM>(st, b);
        }
    }
    if (!dma && ((tile >= 5 && tile <= 8) || tile == 10)) tile = tile == 6 ? 2 : tile == 7 ? 1 : 4;   // register-staged instead
    switch (tile) {
        case 1: return launch_one<128, 128, EPI, AFORM, WFORM, 4>(st, g);
        case 2: return launch_one<128, 256, EPI, AFORM, WFORM, 4>(st, g);
        case 3: return launch_one<256, 256, EPI, AFORM, WFORM, 4>(st, g);
        case 4: return launch_one<256, 256, EPI, AFORM, WFORM, 8>(st, g);
        case 5: if (DMA_OK) return launch_dma<256, 256, EPI, 8, 2>(st, g); break;
        case 6: if (DMA_OK) return launch_dma<128, 256, EPI, 8, 2>(st, g); break;
        case 7: if (DMA_OK) return launch_dma<128, 128, EPI, 4, 2>(st, g); break;
        case 8: if (DMA_OK && EPI != EPI_SWIGLU_BF16) return launch_dma<256, 192, NOSWIGLU, 8, 4>(st, g); break;
        case 9: if (DMA_OK) return spk_launch_gemm_skinny(st, EPI, g); break;
        case 10: if (DMA_OK && EPI != EPI_SWIGLU_BF16) return launch_dma<256, 320, NOSWIGLU, 8, 4>(st, g); break;
        case 11: if (DMA_OK) return spk_launch_gemm_skinny(st, EPI, g, 16); break;
        case 12: if (DMA_OK) return spk_launch_gemm_skinny(st, EPI, g, 32); break;
        case 13: if (DMA_OK) return spk_launch_gemm_skinny(st, EPI, g, 64); break;
    }
    return hipErrorInvalidValue;
}

}  // namespace

GemmPlan spk_gemm_plan_host(int epi, int a_form, int w_form, int M, int N) {
    return plan_gemm(epi, a_form == OP_KMAJOR && w_form == OP_KMAJOR, M, N);
}

hipError_t spk_launch_gemm(hipStream_t st, int epi, const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    if (g.K <= 0 || g.K % BK || g.N % 8 || g.lda % 8 || g.ldw % 8 || !g.A || !g.W || !g.C) return hipErrorInvalidValue;
    if (((uintptr_t)g.A | (uintptr_t)g.W | (uintptr_t)g.C | (uintptr_t)g.R | (uintptr_t)g.bias) & 15) return hipErrorInvalidValue;
    if (g.ldc % 4 || (epi == EPI_RESID_F32 && (!g.R || g.ldr % 4))) return hipErrorInvalidValue;
    if (g.a_form == OP_RMAJOR && (g.M < 8 || g.M % 8)) return hipErrorInvalidValue;
    if (g.w_form == OP_RMAJOR && (g.N < 8 || g.N % 8)) return hipErrorInvalidValue;
    const int forms = g.a_form * 2 + g.w_form;
    switch (epi) {
        case EPI_BF16:
            if (forms == 0) return launch_tile<EPI_BF16, OP_KMAJOR, OP_KMAJOR>(st, g);
            if (forms == 1) return launch_tile<EPI_BF16, OP_KMAJOR, OP_RMAJOR>(st, g);
            break;
        case EPI_RESID_F32:
            if (forms == 0) return launch_tile<EPI_RESID_F32, OP_KMAJOR, OP_KMAJOR>(st, g);
            if (forms == 1) return launch_tile<EPI_RESID_F32, OP_KMAJOR, OP_RMAJOR>(st, g);
            break;
        case EPI_GELU_BF16:
            if (forms == 0 && g.bias) return launch_tile<EPI_GELU_BF16, OP_KMAJOR, OP_KMAJOR>(st, g);
            break;
        case EPI_SWIGLU_BF16:
            if (forms == 0 && !g.bias) return launch_tile<EPI_SWIGLU_BF16, OP_KMAJOR, OP_KMAJOR>(st, g);
            break;
        case EPI_F32:
            if (forms == 1) return launch_tile<EPI_F32, OP_KMAJOR, OP_RMAJOR>(st, g);
            if (forms == 3) return launch_tile<EPI_F32, OP_RMAJOR, OP_RMAJOR>(st, g);
            if (forms == 0) return launch_tile<EPI_F32, OP_KMAJOR, OP_KMAJOR>(st, g);
            break;
    }
    return hipErrorInvalidValue;
}
