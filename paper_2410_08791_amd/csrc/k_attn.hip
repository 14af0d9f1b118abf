// Attention forward: o = softmax(q k^T / sqrt(hd) + mask) v per (batch, head),
// causal or bidirectional, grouped-query heads, head_dim in {64, 80, 128}.
//
// One work-group (4 waves) handles 128 queries of one head; a wave owns 32 of
// them.  Keys/values stream through LDS in tiles of 64.  Scores are computed
// TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in the accumulator
// layout a lane then holds ONE query (its column) and 16 keys of each 32-key
// tile, so the softmax row maximum and sum are in-lane reductions plus one
// exchange between the two half-waves, and the probabilities -- rounded to
// bf16 in place -- already sit in the B-operand layout of the second product
// O^T = V^T P^T.  (The contraction order over keys inside a 16-key MFMA step is
// a fixed permutation; V^T fragments are fetched with the same permutation.)
// V tiles are staged as they lie in memory (one row per key) and the V^T
// fragments come out of the transposing LDS read ds_read_b64_tr_b16, which hands
// a lane four consecutive keys of one head_dim element: no transposed copy of V
// exists anywhere.
//
// K and V tiles go from global memory straight into LDS (global_load_lds_dwordx4,
// issued one tile ahead into the other stage): no staging registers, no ds_write.  A wave
// instruction lands 1 KiB contiguously, so rows cannot be padded against bank conflicts;
// the 16-byte chunks of a row are XOR-swizzled instead, on the global side (which chunk a
// lane fetches).  Rows are 2*head_dim bytes (head_dim 80: 192, the lanes that land in the
// padding fetch a dummy chunk).  K rows: chunk ^ (row & 15) for 256-byte rows,
// ^ ((row >> 1) & 7) for 128, ^ ((row >> 2) & 3) for 192 -- the 16 rows a ds_read_b128 serves
// at a time then cover all banks.  V rows: the 64-byte block (one 32-element tile of O^T)
// ^ (row & 3) for 256-byte rows, ^ ((row >> 1) & 1) for 128, none for 192 -- the four key
// rows of a transposing read fall into different bank groups.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int QB = 128;   // queries per work-group
constexpr int KB = 64;    // keys per LDS tile
constexpr int PF = 3;     // fragment reads in flight ahead of the MFMA that uses them

template <int HD>
struct AttnCfg {
    static constexpr int NKS = HD / 16;             // MFMA k-steps over head_dim
    static constexpr int NMT = (HD + 31) / 32;      // 32-row tiles of O^T
    static constexpr int HDP = NMT * 32;
    static constexpr int ROWB = HD == 80 ? 192 : HD * 2;   // bytes per key / value row in LDS
    static constexpr int CPR = HD / 8;                     // 16-byte chunks of a row that hold data
    static constexpr int TILE_BYTES = KB * ROWB;           // one K or one V tile
    static constexpr int STAGE = 2 * TILE_BYTES;           // K tile, then V tile
    static constexpr int NLOAD = STAGE / 1024 / 4;         // load instructions per wave and stage
    static_assert(STAGE % 4096 == 0 && TILE_BYTES % 1024 == 0, "whole load instructions per wave and per tile");
    static_assert(HDP * 2 <= ROWB, "the fragment reads of a padded head_dim stay inside the row");
    __device__ static int k_swz(int row) { return HD == 128 ? (row & 15) : HD == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
    // in 64-byte blocks
    __device__ static int v_swz(int row) { return HD == 128 ? (row & 3) : HD == 64 ? ((row >> 1) & 1) : 0; }
};

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr_a;

template <int HD>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                       bf16_t* __restrict__ o, float* __restrict__ lse,
                                                       int S, int Hq, int Hkv, int ld_qkv,
                                                       int causal, int paired, float scale_log2e) {
    typedef AttnCfg<HD> C;
    // two stages of {K tile, V tile}
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    // Causal: query block i walks i + 1 key tiles of 128.  With `paired` a work-group takes the
    // blocks nqb - 1 - i and i one after the other, so that every work-group has the same amount
    // of work (gridDim.x = ceil(nqb / 2)); the launcher asks for that when it still leaves two
    // work-groups per CU.  Otherwise one block per work-group: ids are dealt to the CUs in
    // order, two resident per CU, and every other batch of 256 ids walks the query blocks in
    // the opposite direction, so a CU holds one heavy and one light block.
    const int nqb = (S + QB - 1) / QB;
    const int h = blockIdx.y, b = blockIdx.z;
    const int kvh = h / (Hq / Hkv);
    const int bx = blockIdx.x;
    const int lin = bx + (int)gridDim.x * (h + (int)gridDim.y * b);
    const int nphase = (paired && nqb - 1 - bx != bx) ? 2 : 1;
    const size_t tok0 = (size_t)b * S;
    const bf16_t* kbase = qkv + tok0 * ld_qkv + (size_t)Hq * HD + (size_t)kvh * HD;
    const bf16_t* vbase = kbase + (size_t)Hkv * HD;
    // load assignment: instruction i of this wave lands at byte (wave * NLOAD + i) * 1024 + lane * 16
    // of a stage; the lane fetches the chunk that the swizzle puts there
    const bf16_t* ld_col[C::NLOAD];
    int ld_row[C::NLOAD];
#pragma unroll
    for (int i = 0; i < C::NLOAD; ++i) {
        const int off = (wave * C::NLOAD + i) * 1024 + lane * 16;
        const bool isv = off >= C::TILE_BYTES;
        const int rel = off - (isv ? C::TILE_BYTES : 0);
        const int row = rel / C::ROWB, pos = (rel % C::ROWB) >> 4;
        int c = isv ? pos ^ (C::v_swz(row) << 2) : pos ^ C::k_swz(row);
        if (c >= C::CPR) c = 0;                       // padding of the 192-byte rows: any valid chunk
        ld_row[i] = row;
        ld_col[i] = (isv ? vbase : kbase) + c * 8;
    }
#if defined(__HIP_DEVICE_COMPILE__)
#define SP_ATTN_ISSUE(kt_, stage_)                                                                             \
    do {                                                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < C::NLOAD; ++i_)                                                \
            __builtin_amdgcn_global_load_lds(ld_col[i_] + (size_t)min((kt_) * KB + ld_row[i_], S - 1) * ld_qkv, \
                                             (lds_void_ptr_a)(smem_attn + (stage_) * C::STAGE +                \
                                                              (wave * C::NLOAD + i_) * 1024), 16, 0, 0);      \
    } while (0)
#else
#define SP_ATTN_ISSUE(kt_, stage_) ((void)ld_col, (void)ld_row)
#endif
    constexpr int WAIT_VM0 = (0 & 15) | (7 << 4) | (15 << 8) | (0 << 14);   // vmcnt 0, lgkmcnt untouched
    // fragment addresses inside a tile (the swizzle terms depend on the lane only)
    int kpos[C::NKS];
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks) kpos[ks] = l32 * C::ROWB + (((2 * ks + half) ^ C::k_swz(l32)) << 4);
    int vpos[C::NMT];
    {
        const int rowv = half * 4 + ((lane & 15) >> 2);
#pragma unroll
        for (int mt = 0; mt < C::NMT; ++mt)
            vpos[mt] = rowv * C::ROWB + ((mt ^ C::v_swz(rowv)) << 6) + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);
    }
    for (int phase = 0; phase < nphase; ++phase) {
    const int qb = paired ? (phase ? bx : nqb - 1 - bx)                          // heavy block first
                          : (!causal || ((lin >> 8) & 1)) ? bx : nqb - 1 - bx;
    const int q0 = qb * QB;
    const int wq0 = q0 + wave * 32;          // this wave's first query
    const int qi = wq0 + l32;                // this lane's query

    // Q fragments: B operand, column = query, 8 contiguous head_dim elements.
    bf16x8_t qf[C::NKS];
    {
        const int qr = min(qi, S - 1);
        const bf16_t* qp = qkv + (tok0 + qr) * ld_qkv + h * HD + half * 8;
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16);
    }

    f32x16_t oacc[C::NMT];
#pragma unroll
    for (int t = 0; t < C::NMT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[t][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int k_end = causal ? min(S, q0 + QB) : S;
    const int ntiles = (k_end + KB - 1) / KB;
    const int wq_last = wq0 + 31;

    // Tile kt+1 is loaded into stage (kt+1)&1 while stage kt&1 is consumed; one barrier per tile.
    SP_ATTN_ISSUE(0, 0);
    __builtin_amdgcn_s_waitcnt(WAIT_VM0);
    asm volatile("" ::: "memory");
    __syncthreads();

    for (int kt = 0; kt < ntiles; ++kt) {
        const int key0 = kt * KB;
        const bool more = kt + 1 < ntiles;
        if (more) SP_ATTN_ISSUE(kt + 1, (kt + 1) & 1);
        const unsigned char* sK = smem_attn + (kt & 1) * C::STAGE;
        const unsigned char* sV = sK + C::TILE_BYTES;
        // wave-uniform skips: nothing visible to this wave / no valid query in this wave
        if (!((causal && key0 > wq_last) || wq0 >= S)) {

        // ---- S^T = K Q^T for two 32-key tiles.  The K fragments are read PF steps ahead of the
        //      MFMA that consumes them (scheduling hints keep the compiler from sinking a read
        //      down to its use, which would expose the LDS latency before every MFMA), and
        //      consecutive MFMAs alternate between the two tiles' accumulators.
        f32x16_t sacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[t][e] = 0.f;
        {
            constexpr int NQK = 2 * C::NKS;
            bf16x8_t kf[NQK];
            auto kread = [&](int st) {   // step st: tile st & 1, k-step st >> 1
                kf[st] = *reinterpret_cast<const bf16x8_t*>(sK + (st & 1) * 32 * C::ROWB + kpos[st >> 1]);
            };
#pragma unroll
            for (int st = 0; st < PF; ++st) kread(st);
#pragma unroll
            for (int st = 0; st < NQK; ++st) {
                if (st + PF < NQK) kread(st + PF);
                sacc[st & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st], qf[st >> 1], sacc[st & 1], 0, 0, 0);
            }
            // issue order: PF reads, then one read per MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
#pragma unroll
            for (int st = 0; st < NQK; ++st) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (st + PF < NQK) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        // V^T fragments of step st = (t, j, mt): tile mt of O^T, keys of (t, j)
        constexpr int NPV = 4 * C::NMT;
        typedef short s16x8_t __attribute__((ext_vector_type(8)));
        s16x8_t vf[NPV];
        auto vread = [&](int st) {
            const int tj = st / C::NMT, mt = st % C::NMT;
            const unsigned char* vp = sV + ((tj >> 1) * 32 + 16 * (tj & 1)) * C::ROWB + vpos[mt];
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp + 8 * C::ROWB));
            vf[st] = s16x8_t{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        };
#pragma unroll
        for (int st = 0; st < PF; ++st) vread(st);
        asm volatile("" ::: "memory");
        // ---- mask, online softmax in base 2 on the raw scores (the scale is positive,
        //      so it commutes with max and is folded into the exponent's fma)
        const bool need_mask = (causal && key0 + KB - 1 > wq0) || (key0 + KB > S);
        float mx = -INFINITY;
        if (need_mask) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + t * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                    if (key >= S || (causal && key > qi)) sacc[t][e] = -INFINITY;
                }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[t][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // The reference maximum m_run follows the true one lazily: it moves only when a score
        // exceeds it by more than 2^8 in the exponent.  Probabilities are then at most 256
        // instead of 1 (bf16 has the range, the denominator and O^T are fp32, and both carry the
        // same reference), and the rescale of O^T below -- 16 multiplies per MFMA tile --
        // becomes rare instead of running in nearly every tile.
        const bool move = (mx - m_run) * scale_log2e > 8.0f;   // first tile: m_run = -inf, mx finite (key 0 is visible to every query)
        const float m_new = move ? mx : m_run;
        const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e) : 1.0f;
        const float m_scaled = m_new * scale_log2e;
        m_run = m_new;
        float psum = 0.f;
        bf16x8_t pf[2][2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[t][j * 8 + e], scale_log2e, -m_scaled));
                    psum += pv;
                    pf[t][j][e] = (__bf16)pv;
                }
        l_run = l_run * alpha + psum;
        if (__any(move)) {   // the reference moved for some query of the wave
#pragma unroll
            for (int t = 0; t < C::NMT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
        }
        // ---- O^T += V^T P^T.  Step (t, j) contracts keys
        //      t*32 + 16j + {half*4 + 0..3, 8 + half*4 + 0..3}.  The transposing read works on
        //      groups of 16 lanes: lane s of a group points at key row (s>>2) of the step's four
        //      and at 4 head_dim elements, and receives four consecutive keys of ITS element
        //      (16 * (group & 1) + s within the 32-row tile).  Fragments are read PF steps ahead
        //      (the first PF before the softmax arithmetic above, which hides their latency);
        //      consecutive MFMAs go to different 32-row tiles of O^T.
#pragma unroll
        for (int st = 0; st < NPV; ++st) {
            if (st + PF < NPV) vread(st + PF);
            const int tj = st / C::NMT, mt = st % C::NMT;
            oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[st]),
                                                               pf[tj >> 1][tj & 1], oacc[mt], 0, 0, 0);
        }
#pragma unroll
        for (int st = 0; st < NPV; ++st) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (st + PF < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        }
        // this wave's loads of tile kt+1 have landed; after the barrier every wave's have, and
        // every wave is done reading stage kt&1
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        asm volatile("" ::: "memory");
        __syncthreads();
    }

    // ---- finish: denominators, write o (and the log-sum-exp for the backward)
    l_run += __shfl_xor(l_run, 32, 64);
    if (qi < S) {
        const float inv = 1.0f / l_run;
        bf16_t* op = o + (tok0 + qi) * (size_t)(Hq * HD) + h * HD;
#pragma unroll
        for (int mt = 0; mt < C::NMT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e0 = mt * 32 + g * 8 + half * 4;
                if (e0 < HD)
                    *reinterpret_cast<uint2*>(op + e0) =
                        make_uint2(pack_bf2(oacc[mt][g * 4] * inv, oacc[mt][g * 4 + 1] * inv),
                                   pack_bf2(oacc[mt][g * 4 + 2] * inv, oacc[mt][g * 4 + 3] * inv));
            }
        if (lse && half == 0)
            lse[((size_t)b * Hq + h) * S + qi] = m_run * scale_log2e * 0.69314718055994530942f + logf(l_run);
    }
    }   // phase
#undef SP_ATTN_ISSUE
}

template <int HD>
hipError_t launch_fwd(hipStream_t st, dim3 grid, const bf16_t* qkv, bf16_t* o, float* lse,
                      const AttnShape& a, int paired, float sl2) {
    typedef AttnCfg<HD> C;
    constexpr int LDS = 2 * C::STAGE;
    static LdsLimitOnce lds_limit;
    hipError_t e = lds_limit.set(reinterpret_cast<const void*>(attn_fwd_kernel<HD>), LDS);
    if (e != hipSuccess) return e;
    attn_fwd_kernel<HD><<<grid, 256, LDS, st>>>(qkv, o, lse, a.S, a.Hq, a.Hkv, a.ld_qkv, a.causal, paired, sl2);
    return hipGetLastError();
}

}  // namespace

hipError_t spk_launch_attention(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a) {
    if (a.B <= 0 || a.S <= 0) return hipSuccess;
    if (a.Hkv <= 0 || a.Hq % a.Hkv || a.ld_qkv % 8 || a.B > 65535 || a.Hq > 65535) return hipErrorInvalidValue;
    if (((uintptr_t)qkv | (uintptr_t)o) & 15) return hipErrorInvalidValue;
    const float sl2 = 1.4426950408889634f / sqrtf((float)a.hd);
    const int nqb = (a.S + QB - 1) / QB;
    const int paired = a.causal && (long)((nqb + 1) / 2) * a.Hq * a.B >= 512;
    dim3 grid(paired ? (nqb + 1) / 2 : nqb, a.Hq, a.B);
    switch (a.hd) {
        case 64: return launch_fwd<64>(st, grid, qkv, o, lse, a, paired, sl2);
        case 80: return launch_fwd<80>(st, grid, qkv, o, lse, a, paired, sl2);
        case 128: return launch_fwd<128>(st, grid, qkv, o, lse, a, paired, sl2);
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
