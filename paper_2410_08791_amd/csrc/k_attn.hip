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

constexpr int KB = 64;    // keys per LDS tile
constexpr int PF = 3;     // fragment reads in flight ahead of the MFMA that uses them

// NW = waves per work-group: a work-group handles NW * 32 queries of one head.
template <int HD, int NW>
struct AttnCfg {
    static constexpr int QB = NW * 32;              // queries per work-group
    static constexpr int NKS = HD / 16;             // MFMA k-steps over head_dim
    static constexpr int NMT = (HD + 31) / 32;      // 32-row tiles of O^T
    static constexpr int HDP = NMT * 32;
    static constexpr int ROWB = HD == 80 ? 192 : HD * 2;   // bytes per key / value row in LDS
    static constexpr int CPR = HD / 8;                     // 16-byte chunks of a row that hold data
    static constexpr int TILE_BYTES = KB * ROWB;           // one K or one V tile
    static constexpr int STAGE = 2 * TILE_BYTES;           // K tile, then V tile
    static constexpr int NINST = STAGE / 1024;             // 1 KiB load instructions per stage
    static constexpr int NLOAD = (NINST + NW - 1) / NW;    // per wave (the last wave may have fewer)
    // head_dim 80: the rows 80..95 of the third O^T tile are padding.  The V tiles' padding
    // elements are set to 1.0 once and never loaded over, so row 80 of O^T accumulates the sum of
    // the (bf16) probabilities: the softmax denominator comes out of the matrix pipe, which idles
    // most of the time here, instead of 32 additions per lane and tile on the vector pipe, which
    // is the one that bounds this kernel.
    static constexpr bool ONES_ROW = HDP > HD;
    static_assert(STAGE % 1024 == 0 && TILE_BYTES % 1024 == 0, "whole load instructions per tile");
    static_assert(HDP * 2 <= ROWB, "the fragment reads of a padded head_dim stay inside the row");
    __device__ static int k_swz(int row) { return HD == 128 ? (row & 15) : HD == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
    // in 64-byte blocks
    __device__ static int v_swz(int row) { return HD == 128 ? (row & 3) : HD == 64 ? ((row >> 1) & 1) : 0; }
};

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr_a;

struct SoftmaxState {
    float m_run, l_run;
};

// One key tile for one wave: NT = 32-key halves of the tile that hold keys (2, or 1 for a ragged
// last tile with at most 32 keys left -- S = 257 ends in a tile of one key).
template <int HD, int NW, int NT>
__device__ __forceinline__ void attn_tile(const unsigned char* sK, const unsigned char* sV, const int* kpos,
                                          const int* vpos, const bf16x8_t* qf, f32x16_t* oacc, SoftmaxState& sm,
                                          int key0, int S, int causal, int qi, int wq0, int half, float scale_log2e,
                                          bool first) {
    typedef AttnCfg<HD, NW> C;
    // ---- S^T = K Q^T for NT 32-key tiles.  The K fragments are read PF steps ahead of the
    //      MFMA that consumes them (scheduling hints keep the compiler from sinking a read
    //      down to its use, which would expose the LDS latency before every MFMA), and
    //      consecutive MFMAs alternate between the tiles' accumulators.
    f32x16_t sacc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[t][e] = 0.f;
    {
        constexpr int NQK = NT * C::NKS;
        bf16x8_t kf[NQK];
        auto kread = [&](int st) {   // step st: tile st % NT, k-step st / NT
            kf[st] = *reinterpret_cast<const bf16x8_t*>(sK + (st % NT) * 32 * C::ROWB + kpos[st / NT]);
        };
#pragma unroll
        for (int st = 0; st < PF; ++st) kread(st);
#pragma unroll
        for (int st = 0; st < NQK; ++st) {
            if (st + PF < NQK) kread(st + PF);
            sacc[st % NT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st], qf[st / NT], sacc[st % NT], 0, 0, 0);
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
    constexpr int NPV = 2 * NT * C::NMT;
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
    const bool need_mask = (causal && key0 + NT * 32 - 1 > wq0) || (key0 + NT * 32 > S);
    float mx = -INFINITY;
    if (need_mask) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = key0 + t * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                if (key >= S || (causal && key > qi)) sacc[t][e] = -INFINITY;
            }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[t][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The reference maximum m_run follows the true one lazily: it moves only when a score
    // exceeds it by more than 2^8 in the exponent.  Probabilities are then at most 256
    // instead of 1 (bf16 has the range, the denominator and O^T are fp32, and both carry the
    // same reference), and the rescale of O^T below -- 16 multiplies per MFMA tile --
    // becomes rare instead of running in nearly every tile.
    const bool move = (mx - sm.m_run) * scale_log2e > 8.0f;   // first tile: m_run = -inf, mx finite (key 0 is visible to every query)
    const float m_new = move ? mx : sm.m_run;
    const float alpha = move ? __builtin_amdgcn_exp2f((sm.m_run - m_new) * scale_log2e) : 1.0f;
    const float m_scaled = m_new * scale_log2e;
    sm.m_run = m_new;
    float psum = 0.f;
    bf16x8_t pf[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[t][j * 8 + e], scale_log2e, -m_scaled));
                if (!C::ONES_ROW) psum += pv;
                pf[t][j][e] = (__bf16)pv;
            }
    if (!C::ONES_ROW) sm.l_run = sm.l_run * alpha + psum;
    // the reference moved for some query of the wave; in the first tile O^T is still zero
    if (!first && __any(move)) {
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
        oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[st]), pf[tj >> 1][tj & 1],
                                                           oacc[mt], 0, 0, 0);
    }
#pragma unroll
    for (int st = 0; st < NPV; ++st) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (st + PF < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
}

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ o, float* __restrict__ lse,
                                                            int S, int Hq, int Hkv, int ld_qkv,
                                                            int causal, int paired, float scale_log2e) {
    typedef AttnCfg<HD, NW> C;
    constexpr int QB = C::QB;
    // two stages of {K tile, V tile}
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_attn[];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    // Causal: query block i walks the key tiles up to its own diagonal.  With `paired` a work-group
    // takes the blocks nqb - 1 - i and i one after the other, so that every work-group has the same
    // amount of work (gridDim.x = ceil(nqb / 2)); the launcher asks for that when it still leaves two
    // work-groups per CU.  Otherwise one block per work-group: ids are dealt to the CUs in
    // order, two resident per CU, and every other batch of 256 ids walks the query blocks in
    // the opposite direction, so a CU holds one heavy and one light block.
    const int nqb = (S + QB - 1) / QB;
    // The hardware deals consecutive work-group ids round-robin over the 8 XCDs, each with its own
    // L2.  Ids are remapped so that an XCD works through a contiguous range of (batch, head, query
    // block): every query block of a head -- and every query head of a key/value group -- then
    // reads that head's keys and values through the same L2 instead of fetching them once per XCD.
    const int lin = blockIdx.x + (int)gridDim.x * (blockIdx.y + (int)gridDim.y * blockIdx.z);   // dispatch order
    const int job = xcd_remap(lin, (int)(gridDim.x * gridDim.y * gridDim.z));
    const int bx = job % (int)gridDim.x, h = (job / (int)gridDim.x) % (int)gridDim.y;
    const int b = job / (int)(gridDim.x * gridDim.y);
    const int kvh = h / (Hq / Hkv);
    const int nphase = (paired && nqb - 1 - bx != bx) ? 2 : 1;
    const size_t tok0 = (size_t)b * S;
    const bf16_t* kbase = qkv + tok0 * ld_qkv + (size_t)Hq * HD + (size_t)kvh * HD;
    // load assignment: instruction i of this wave lands at byte (wave * NLOAD + i) * 1024 + lane * 16
    // of a stage; the lane fetches the chunk that the swizzle puts there.  Lanes that land in the
    // padding of the 192-byte rows (head_dim 80) load nothing: what lies there is never read in a K
    // tile and stays 1.0 in a V tile (ONES_ROW).
    int ld_col[C::NLOAD];          // element offset from kbase (the V part lies Hkv * HD further)
    int ld_row[C::NLOAD];
    bool ld_on[C::NLOAD];
#pragma unroll
    for (int i = 0; i < C::NLOAD; ++i) {
        const int off = (wave * C::NLOAD + i) * 1024 + lane * 16;
        const bool isv = off >= C::TILE_BYTES;
        const int rel = off - (isv ? C::TILE_BYTES : 0);
        const int row = rel / C::ROWB, pos = (rel % C::ROWB) >> 4;
        const int c = isv ? pos ^ (C::v_swz(row) << 2) : pos ^ C::k_swz(row);
        ld_on[i] = c < C::CPR;
        ld_row[i] = row;
        ld_col[i] = (isv ? Hkv * HD : 0) + (c < C::CPR ? c : 0) * 8;
    }
#if defined(__HIP_DEVICE_COMPILE__)
#define SP_ATTN_ISSUE(kt_, stage_)                                                                                 \
    do {                                                                                                           \
        _Pragma("unroll") for (int i_ = 0; i_ < C::NLOAD; ++i_)                                                    \
            if (wave * C::NLOAD + i_ < C::NINST && ld_on[i_])                                                      \
                __builtin_amdgcn_global_load_lds(kbase + ((size_t)min((kt_) * KB + ld_row[i_], S - 1) * ld_qkv + ld_col[i_]), \
                                                 (lds_void_ptr_a)(smem_attn + (stage_) * C::STAGE +                \
                                                                  (wave * C::NLOAD + i_) * 1024), 16, 0, 0);      \
    } while (0)
#else
#define SP_ATTN_ISSUE(kt_, stage_) ((void)ld_col, (void)ld_row, (void)ld_on, (void)kbase)
#endif
    constexpr int WAIT_VM0 = (0 & 15) | (7 << 4) | (15 << 8) | (0 << 14);   // vmcnt 0, lgkmcnt untouched
    if (C::ONES_ROW) {
        // the padding elements of every V row, both stages: bf16 1.0
        constexpr int PADB = C::ROWB - HD * 2;                  // bytes per row, a multiple of 16
        constexpr int PER_ROW = PADB / 16;
        for (int i = threadIdx.x; i < 2 * KB * PER_ROW; i += NW * 64) {
            const int stage = i / (KB * PER_ROW), r = (i / PER_ROW) % KB, c = i % PER_ROW;
            *reinterpret_cast<u32x4_t*>(smem_attn + stage * C::STAGE + C::TILE_BYTES + r * C::ROWB + HD * 2 + c * 16) =
                u32x4_t{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
        }
    }
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
    SoftmaxState sm{-INFINITY, 0.f};

    const int k_end = causal ? min(S, q0 + QB) : S;
    const int ntiles = (k_end + KB - 1) / KB;
    const int wq_last = wq0 + 31;

    // Tile kt+1 is loaded into stage (kt+1)&1 while stage kt&1 is consumed; one barrier per tile.
    SP_ATTN_ISSUE(0, 0);
    __builtin_amdgcn_s_waitcnt(WAIT_VM0);
    asm volatile("" ::: "memory");
    __syncthreads();

    // A ragged last tile with at most 32 keys (S = 257 ends in a tile of one key) is worked as
    // one 32-key half, after the loop: its loads and barrier run in the loop like any tile's.
    const bool half_last = HD != 128 && k_end - (ntiles - 1) * KB <= 32;
    for (int kt = 0; kt < ntiles; ++kt) {
        const int key0 = kt * KB;
        const bool more = kt + 1 < ntiles;
        if (more) SP_ATTN_ISSUE(kt + 1, (kt + 1) & 1);
        const unsigned char* sK = smem_attn + (kt & 1) * C::STAGE;
        const unsigned char* sV = sK + C::TILE_BYTES;
        // wave-uniform skips: nothing visible to this wave / no valid query in this wave
        if (!((causal && key0 > wq_last) || wq0 >= S || (half_last && !more)))
            attn_tile<HD, NW, 2>(sK, sV, kpos, vpos, qf, oacc, sm, key0, S, causal, qi, wq0, half, scale_log2e, kt == 0);
        // this wave's loads of tile kt+1 have landed; after the barrier every wave's have, and
        // every wave is done reading stage kt&1
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        asm volatile("" ::: "memory");
        if (more || nphase > 1) __syncthreads();
    }
    if (half_last) {
        const int kt = ntiles - 1, key0 = kt * KB;
        const unsigned char* sK = smem_attn + (kt & 1) * C::STAGE;
        if (!((causal && key0 > wq_last) || wq0 >= S))
            attn_tile<HD, NW, 1>(sK, sK + C::TILE_BYTES, kpos, vpos, qf, oacc, sm, key0, S, causal, qi, wq0, half,
                                 scale_log2e, kt == 0);
        if (nphase > 1) __syncthreads();      // the next phase's first loads overwrite stage 0
    }

    // ---- finish: denominators, write o (and the log-sum-exp for the backward)
    float l_run;
    if (C::ONES_ROW) {
        l_run = oacc[C::NMT - 1][(HD % 32) / 8 * 4];     // row HD of O^T: the sum of the probabilities
    } else {
        l_run = sm.l_run + __shfl_xor(sm.l_run, 32, 64);
    }
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
            lse[((size_t)b * Hq + h) * S + qi] = sm.m_run * scale_log2e * 0.69314718055994530942f + logf(l_run);
    }
    }   // phase
#undef SP_ATTN_ISSUE
}

template <int HD, int NW>
hipError_t launch_fwd(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a, float sl2) {
    typedef AttnCfg<HD, NW> C;
    constexpr int LDS = 2 * C::STAGE;
    static LdsLimitOnce lds_limit;
    hipError_t e = lds_limit.set(reinterpret_cast<const void*>(attn_fwd_kernel<HD, NW>), LDS);
    if (e != hipSuccess) return e;
    const int nqb = (a.S + C::QB - 1) / C::QB;
    const int paired = a.causal && (long)((nqb + 1) / 2) * a.Hq * a.B >= 512;
    dim3 grid(paired ? (nqb + 1) / 2 : nqb, a.Hq, a.B);
    attn_fwd_kernel<HD, NW><<<grid, NW * 64, LDS, st>>>(qkv, o, lse, a.S, a.Hq, a.Hkv, a.ld_qkv, a.causal, paired, sl2);
    return hipGetLastError();
}

// Four waves per work-group.  (Three -- 96 queries, which covers S = 257 with nine busy waves
// instead of nine of twelve -- was measured slower, 64 against 59 us on the ViT-H shape: a CU then
// holds nine waves instead of twelve, and hiding the loads' latency matters more than the idle waves.)
template <int HD>
hipError_t launch_hd(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a, float sl2) {
    return launch_fwd<HD, 4>(st, qkv, o, lse, a, sl2);
}

}  // namespace

hipError_t spk_launch_attention(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a) {
    if (a.B <= 0 || a.S <= 0) return hipSuccess;
    if (a.Hkv <= 0 || a.Hq % a.Hkv || a.ld_qkv % 8 || a.B > 65535 || a.Hq > 65535) return hipErrorInvalidValue;
    if (((uintptr_t)qkv | (uintptr_t)o) & 15) return hipErrorInvalidValue;
    const float sl2 = 1.4426950408889634f / sqrtf((float)a.hd);
    switch (a.hd) {
        case 64: return launch_hd<64>(st, qkv, o, lse, a, sl2);
        case 80: return launch_hd<80>(st, qkv, o, lse, a, sl2);
        case 128: return launch_hd<128>(st, qkv, o, lse, a, sl2);
        default: return hipErrorInvalidValue;
    }
}
