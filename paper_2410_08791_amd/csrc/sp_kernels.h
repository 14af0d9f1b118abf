// Host-side launchers of the per-layer kernels (internal to the library).
// Every launcher validates what its kernel and grid assume, enqueues on `st`
// and returns the launch status; none synchronises or allocates.
// Host declarations only: the device helpers live in sp_common.h, which the kernel sources
// include themselves, so that the engine's host code builds against the HIP runtime API alone.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "sp_limits.h"
#include "sp_types.h"

// Raises a kernel's dynamic-LDS limit once per process; safe when two host threads launch the
// same kernel for the first time together.  Every call returns the status of that one attempt.
struct LdsLimitOnce {
    std::once_flag flag;
    hipError_t status = hipSuccess;
    hipError_t set(const void* kernel, int bytes) {
        std::call_once(flag, [&] {
            status = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        });
        return status;
    }
};

enum GemmEpilogue {
    EPI_BF16 = 0,        // C bf16 [M,N]  = acc (+ bias)
    EPI_RESID_F32 = 1,   // C fp32 [M,N]  = R + acc (+ bias); C may alias R
    EPI_GELU_BF16 = 2,   // C bf16 [M,N]  = gelu(acc + bias), exact erf form
    EPI_SWIGLU_BF16 = 3, // W = [gate rows; up rows] (2N x K); C bf16 [M,N] = silu(gate) * up
    EPI_F32 = 4          // C fp32 [M,N]  = acc (+ bias)   (weight gradients)
};

// Operand forms: which index is contiguous in memory.
//   OP_KMAJOR: element (row r, contraction index k) at ptr[r * ld + k]
//   OP_RMAJOR: element (r, k) at ptr[k * ld + r]   (transposed on the way into LDS)
enum GemmOperand { OP_KMAJOR = 0, OP_RMAJOR = 1 };

struct GemmArgs {
    const bf16_t* A; int lda; int a_form;   // "activation" operand, rows = M
    const bf16_t* W; int ldw; int w_form;   // "weight" operand, rows = N
    void* C; int ldc;
    const float* R; int ldr;                // EPI_RESID_F32
    const bf16_t* bias;                     // [N] or nullptr
    int M, N, K;
    int tile;                               // 0 = heuristic, else 1..9 = forced kernel and tile shape
};

// C[M,N] = sum_k A(m,k) W(n,k), bf16 operands, fp32 accumulate on MFMA.
// Needs K % 64 == 0, N % 8 == 0, leading dimensions % 8 == 0, 16-byte aligned bases.
hipError_t spk_launch_gemm(hipStream_t st, int epilogue, const GemmArgs& g);
// The kernel for at most SPK_SKINNY_MAX_ROWS activation rows (tile id 9; both operands
// contraction-contiguous): streams W once, 16 output columns per work-group, one to four tiles of
// 16 rows per weight fragment.
constexpr int SPK_SKINNY_MAX_ROWS = 64;
hipError_t spk_launch_gemm_skinny(hipStream_t st, int epilogue, const GemmArgs& g, int rows_per_group = 0);
// What tile = 0 resolves to for a shape (host code, no launch): rows [0, body_rows) run with
// `tile`, rows [body_rows, M) -- none when body_rows == M -- with `tail_tile`.
struct GemmPlan { int tile, body_rows, tail_tile; };
GemmPlan spk_gemm_plan_host(int epilogue, int a_form, int w_form, int M, int N);

// out bf16 [T,d] = norm(h fp32 [T,d]); bias == nullptr -> RMSNorm, else LayerNorm.
hipError_t spk_launch_norm(hipStream_t st, const float* h, const bf16_t* gain, const bf16_t* bias,
                           bf16_t* out, int T, int d, float eps);

// z bf16 [T,f] = silu(gu[:, :f]) * gu[:, f:], gu bf16 [T,2f].
hipError_t spk_launch_swiglu(hipStream_t st, const bf16_t* gu, bf16_t* z, int T, int f);

struct AttnShape {
    int B, S, Hq, Hkv, hd, causal;
    int ld_qkv;      // row stride (elements) of the fused [q | k | v] activation
};

// o bf16 [B*S, Hq*hd] = softmax(q k^T / sqrt(hd) + mask) v per (batch, head);
// lse (nullable) fp32 [B, Hq, S] = log of the softmax denominator incl. the row max.
hipError_t spk_launch_attention(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a);

// ---- decode (key/value cache) ---------------------------------------------------------
// One layer's cache: kt bf16 [B][Hkv][hd][max_len], v bf16 [B][Hkv][max_len][hd].
// Copies the k and v parts of qkv [B*S, ld_qkv] into positions pos0 .. pos0+S-1.
hipError_t spk_launch_kv_append(hipStream_t st, const bf16_t* qkv, int ld_qkv, bf16_t* kt, bf16_t* v, int B, int S,
                                int pos0, int Hq, int Hkv, int hd, int max_len);
// o bf16 [B, ld_o] = softmax(q K^T / sqrt(hd)) V for one query per sequence (row b of qkv)
// over the first n cached positions.  hd 64 or 128, max_len a multiple of 8 and <= kDecodeMaxLen, kt and v 16-byte aligned.
hipError_t spk_launch_decode_attention(hipStream_t st, const bf16_t* qkv, int ld_qkv, const bf16_t* kt,
                                       const bf16_t* v, bf16_t* o, int ld_o, int B, int n, int max_len, int Hq,
                                       int Hkv, int hd);

hipError_t spk_launch_copy_f32(hipStream_t st, const float* src, float* dst, size_t n);
hipError_t spk_launch_fill_u32(hipStream_t st, uint32_t* dst, uint32_t v, size_t n);
// A one-wave kernel that idles for about `micros` microseconds (at most SPK_SPIN_MAX_US) and exits.
hipError_t spk_launch_spin(hipStream_t st, int micros);

// ---- backward ---------------------------------------------------------------------
// loss = mean((y-t)^2) over n elements; dy = 2(y-t)/n as fp32 and as bf16.  part: SPK_MSE_PARTS floats.
hipError_t spk_launch_mse(hipStream_t st, const float* y, const float* t, float* dy, bf16_t* dyb, float* part,
                          float* loss, size_t n);
// gu = [g | u] bf16 [T,2f] is overwritten by [dg | du] given dz bf16 [T,f].
hipError_t spk_launch_swiglu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* gu, int T, int f);
// RMSNorm backward: dh_io (fp32 [T,d]) += d(norm)/dh applied to da; dhb = bf16(dh_io);
// dgain fp32 [d] = sum_t da*h*r.  part: SPK_NORM_BWD_BLOCKS * d floats.
hipError_t spk_launch_rmsnorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                  bf16_t* dhb, float* part, float* dgain, int T, int d, float eps);
// LayerNorm backward (biased variance): dh_io += d(norm)/dh applied to da; dhb = bf16(dh_io);
// dgain = sum_t da*xhat, dbias = sum_t da.  part: SPK_NORM_BWD_BLOCKS * 2d floats.
hipError_t spk_launch_layernorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                    bf16_t* dhb, float* part, float* dgain, float* dbias, int T, int d, float eps);
// z = gelu(u) (exact-erf form) over n bf16 elements; and u <- dz * gelu'(u) in place.
hipError_t spk_launch_gelu(hipStream_t st, const bf16_t* u, bf16_t* z, size_t n);
hipError_t spk_launch_gelu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* u, size_t n);
// out fp32 [n] = column sums over the T rows of src bf16 [T, ld] (bias gradients).
// part: SPK_NORM_BWD_BLOCKS * n floats.
hipError_t spk_launch_colsum_bf16(hipStream_t st, const bf16_t* src, int ld, int T, int n, float* part, float* out);
hipError_t spk_launch_f32_to_bf16(hipStream_t st, const float* src, bf16_t* dst, size_t n);
// delta fp32 [B,Hq,S] = rowsum(dO * O), both bf16 [B*S, Hq*hd].
hipError_t spk_launch_attn_delta(hipStream_t st, const bf16_t* dO, const bf16_t* O, float* delta, int B, int S,
                                 int Hq, int hd);
// Attention backward.  qkv, dO, lse, delta as produced by the forward / the launchers above;
// Writes dq, dk, dv
// into dqkv (same layout as qkv, bf16).
struct AttnBwdArgs {
    const bf16_t* qkv; const bf16_t* dO; const float* lse; const float* delta;
    bf16_t* dqkv;
};
hipError_t spk_launch_attention_bwd(hipStream_t st, const AttnBwdArgs& g, const AttnShape& a);
