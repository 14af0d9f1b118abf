/*
 * superpipe_kernels.h -- C ABI test hooks for the individual per-layer kernels.
 *
 * These exist so that each kernel can be compared with the CPU oracle's op on
 * its own; the product path is superpipe.h.  All pointers are device (HBM)
 * addresses on the current HIP device, 16-byte aligned; `stream` is a
 * hipStream_t (NULL = default stream).  Calls enqueue and return a sp_status
 * (SP_ERR_INVALID_ARG when the shape is one the kernel does not take,
 * SP_ERR_HIP when the launch fails); nothing is allocated.  bf16 buffers hold
 * raw 16-bit patterns.
 *
 * The operations are the per-layer steps of the streamed stack: the paper's
 * method leaves them unchanged (Sec. 4.2), their definitions are those of a
 * pre-norm transformer layer.
 */
#ifndef SUPERPIPE_KERNELS_H
#define SUPERPIPE_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* out bf16 [T,d] = h * rsqrt(mean(h^2)+eps) * gain          (bias == NULL)
 *               = (h-mean) * rsqrt(var+eps) * gain + bias   (bias != NULL)
 * h fp32 [T,d]; gain/bias bf16 [d]; d % 4 == 0, d <= 8192. */
int spk_norm(void* stream, const float* h, const uint16_t* gain, const uint16_t* bias, uint16_t* out,
             int T, int d, float eps);

/* C[M,N] = sum_k A(m,k) W(n,k), bf16 inputs, fp32 accumulate.
 * epilogue: 0 C bf16 = acc (+bias); 1 C fp32 = R + acc (+bias), C may alias R;
 *           2 C bf16 = gelu(acc + bias); 3 W holds 2N rows [gate; up], C bf16 = silu(gate)*up;
 *           4 C fp32 = acc (+bias).
 * a_form / w_form: 0 = contraction index contiguous (A[m*lda+k], W[n*ldw+k]),
 *                  1 = row index contiguous        (A[k*lda+m], W[k*ldw+n]).
 * tile: 0 = library heuristic; 1..4 force a block tile of the register-staged kernel (128x128, 128x256,
 *       256x256 with 4 waves, 256x256 with 8 waves), 5..8 of the LDS-DMA kernel (256x256, 128x256, 128x128,
 *       256x192 -- the last not with epilogue 3; when an operand has form 1 a register-staged kernel runs
 *       instead), 10 the 256x320 tile of the LDS-DMA kernel (not with epilogue 3), 9 the weight-streaming
 *       kernel for M <= 64 rows (both forms 0; the heuristic's choice for such M: a decode step reads every
 *       weight once and re-uses nothing) with its own choice of rows per work-group, 11 / 12 / 13 the same
 *       kernel with 16 / 32 / 64 rows per work-group (more rows than that become further work-groups on
 *       the same 16 output columns).
 * K % 64 == 0, N % 8 == 0. */
int spk_gemm(void* stream, int epilogue, const uint16_t* A, int lda, int a_form, const uint16_t* W, int ldw,
             int w_form, void* C, int ldc, const float* R, int ldr, const uint16_t* bias, int M, int N, int K,
             int tile);

/* What tile = 0 resolves to for a shape (host-only query, nothing is launched; the choice depends on
 * the shape alone, never on addresses or on the streaming window): out3 (host) = {tile id of rows
 * [0, body_rows), body_rows, tile id of rows [body_rows, M) or 0 when body_rows == M}. */
int spk_gemm_plan(int epilogue, int a_form, int w_form, int M, int N, int* out3);

/* z bf16 [T,f] = silu(gu[:, :f]) * gu[:, f:]; gu bf16 [T,2f]; f % 8 == 0. */
int spk_swiglu(void* stream, const uint16_t* gu, uint16_t* z, int T, int f);

/* Attention over a fused activation qkv bf16 [B*S, (Hq+2Hkv)*hd] (query heads,
 * then key heads, then value heads).  o bf16 [B*S, Hq*hd].  lse fp32 [B,Hq,S] or NULL.  hd in {64,80,128}. */
int spk_attention(void* stream, const uint16_t* qkv, uint16_t* o, float* lse,
                  int B, int S, int Hq, int Hkv, int hd, int causal);

/* ---- decode steps (one new token per sequence against a key/value cache) ---- */

/* One layer's cache: kt bf16 [B][Hkv][hd][max_len] (keys, position contiguous) and
 * v bf16 [B][Hkv][max_len][hd].  Copies the key and value parts of the fused
 * activation qkv bf16 [B*S, (Hq+2Hkv)*hd] into positions pos0 .. pos0+S-1.
 * pos0 + S <= max_len, hd <= 128. */
int spk_kv_append(void* stream, const uint16_t* qkv, uint16_t* kt, uint16_t* v, int B, int S, int pos0,
                  int Hq, int Hkv, int hd, int max_len);

/* o bf16 [B, Hq*hd]: row b = softmax(q_b K^T / sqrt(hd)) V over the first n cached
 * positions of sequence b, q_b = the query part of row b of qkv bf16 [B, (Hq+2Hkv)*hd].
 * hd 64 or 128; max_len a multiple of 8, <= 32768; kt and v 16-byte aligned; 1 <= n <= max_len. */
int spk_decode_attention(void* stream, const uint16_t* qkv, const uint16_t* kt, const uint16_t* v, uint16_t* o,
                         int B, int n, int max_len, int Hq, int Hkv, int hd);

/* ---- backward steps (training, Sec. 3.3) ---- */

/* loss[0] = mean((y-t)^2) over n fp32 elements; dy fp32 [n] = 2 (y-t)/n; dy_bf16 the same rounded.
 * scratch: 1024 floats. */
int spk_mse(void* stream, const float* y, const float* t, float* dy, uint16_t* dy_bf16, float* scratch,
            float* loss, size_t n);

/* gu = [g | u] bf16 [T,2f] is overwritten by [dL/dg | dL/du] given dz bf16 [T,f]. */
int spk_swiglu_bwd(void* stream, const uint16_t* dz, uint16_t* gu, int T, int f);

/* RMSNorm backward.  da fp32 [T,d] = gradient w.r.t. the normed output, h fp32 [T,d] the norm
 * input, gain bf16 [d].  dh_io fp32 [T,d] += gradient w.r.t. h; dh_bf16 = bf16(dh_io);
 * dgain fp32 [d] = sum_t da*h*rsqrt(mean(h^2)+eps).  scratch: 256*d floats. */
int spk_rmsnorm_bwd(void* stream, const float* da, const float* h, const uint16_t* gain, float* dh_io,
                    uint16_t* dh_bf16, float* scratch, float* dgain, int T, int d, float eps);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): spk_rmsnorm_bwd without the scratch argument.  The
 * partial rows live in an array built into the library (4 MiB per device, held until the process
 * ends), so the call allocates nothing; same kernels, same results as spk_rmsnorm_bwd.
 * d % 4 == 0 and d <= spk_rmsnorm_bwd_static_max_d() (4096), else SP_ERR_SHAPE.  All calls on one
 * device share the array: calls that overlap on one device (two streams, two threads) race;
 * calls on one stream are ordered and safe.  The array keeps the previous call's contents and
 * needs no clearing (every row read was written by the same call). */
int spk_rmsnorm_bwd_static_max_d(void);
int spk_rmsnorm_bwd_static(void* stream, const float* da, const float* h, const uint16_t* gain, float* dh_io,
                           uint16_t* dh_bf16, float* dgain, int T, int d, float eps);

/* Attention backward.  qkv as in spk_attention, o and lse its outputs, dO bf16 [B*S, Hq*hd].
 * dqkv bf16 (layout of qkv) receives dq, dk, dv.  scratch: spk_attention_bwd_scratch_bytes bytes
 * (the fp32 row sums of dO * O). */
size_t spk_attention_bwd_scratch_bytes(int B, int S, int Hq, int Hkv, int hd);
int spk_attention_bwd(void* stream, const uint16_t* qkv, const uint16_t* o, const uint16_t* dO, const float* lse,
                      void* scratch, uint16_t* dqkv, int B, int S, int Hq, int Hkv, int hd, int causal);

/* ---- backward steps of the encoder layer ---- */

/* LayerNorm backward (biased variance, as in spk_norm with bias != NULL): given da fp32 [T,d],
 * the norm's input h fp32 [T,d] and gain bf16 [d]:  dh_io fp32 [T,d] += dL/dh;
 * dh_bf16 = the updated dh_io rounded; dgain fp32 [d] = sum_t da*xhat; dbias fp32 [d] = sum_t da.
 * scratch: 256 * 2d floats.  d % 4 == 0, d <= 8192. */
int spk_layernorm_bwd(void* stream, const float* da, const float* h, const uint16_t* gain, float* dh_io,
                      uint16_t* dh_bf16, float* scratch, float* dgain, float* dbias, int T, int d, float eps);

/* z bf16 [n] = gelu(u) (0.5 u (1 + erf(u / sqrt 2))); and the backward in place:
 * u <- dz * gelu'(u).  n % 8 == 0. */
int spk_gelu(void* stream, const uint16_t* u, uint16_t* z, size_t n);
int spk_gelu_bwd(void* stream, const uint16_t* dz, uint16_t* u, size_t n);

/* out fp32 [n] = sum over the T rows of src bf16 [T, ld] (bias gradient of a linear map).
 * scratch: 256 * n floats.  n and ld even. */
int spk_colsum_bf16(void* stream, const uint16_t* src, int ld, int T, int n, float* scratch, float* out);

#ifdef __cplusplus
}
#endif
#endif
