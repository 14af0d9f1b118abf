// C ABI wrappers around the kernel launchers, for per-kernel parity tests.
#include "../../include/superpipe.h"
#include "../../include/superpipe_kernels.h"
#include "sp_kernels.h"

static int st(hipError_t e) {
    if (e == hipSuccess) return SP_OK;
    (void)hipGetLastError();
    return e == hipErrorInvalidValue ? SP_ERR_INVALID_ARG : SP_ERR_HIP;
}

extern "C" int spk_norm(void* stream, const float* h, const uint16_t* gain, const uint16_t* bias, uint16_t* out,
                        int T, int d, float eps) {
    if (!h || !gain || !out) return SP_ERR_INVALID_ARG;
    return st(spk_launch_norm((hipStream_t)stream, h, gain, bias, out, T, d, eps));
}

extern "C" int spk_gemm(void* stream, int epilogue, const uint16_t* A, int lda, int a_form, const uint16_t* W,
                        int ldw, int w_form, void* C, int ldc, const float* R, int ldr, const uint16_t* bias,
                        int M, int N, int K, int tile) {
    if (a_form < 0 || a_form > 1 || w_form < 0 || w_form > 1 || tile < 0 || tile > 13) return SP_ERR_INVALID_ARG;
    GemmArgs g{A, lda, a_form, W, ldw, w_form, C, ldc, R, ldr, bias, M, N, K, tile};
    return st(spk_launch_gemm((hipStream_t)stream, epilogue, g));
}

extern "C" int spk_gemm_plan(int epilogue, int a_form, int w_form, int M, int N, int* out3) {
    if (!out3 || epilogue < 0 || epilogue > 4 || a_form < 0 || a_form > 1 || w_form < 0 || w_form > 1 || M < 1 || N < 1)
        return SP_ERR_INVALID_ARG;
    const GemmPlan pl = spk_gemm_plan_host(epilogue, a_form, w_form, M, N);
    out3[0] = pl.tile; out3[1] = pl.body_rows; out3[2] = pl.tail_tile;
    return SP_OK;
}

extern "C" int spk_swiglu(void* stream, const uint16_t* gu, uint16_t* z, int T, int f) {
    if (!gu || !z) return SP_ERR_INVALID_ARG;
    return st(spk_launch_swiglu((hipStream_t)stream, gu, z, T, f));
}

extern "C" int spk_attention(void* stream, const uint16_t* qkv, uint16_t* o, float* lse, int B, int S, int Hq,
                             int Hkv, int hd, int causal) {
    if (!qkv || !o || B < 1 || S < 1 || Hq < 1 || Hkv < 1) return SP_ERR_INVALID_ARG;
    AttnShape a{B, S, Hq, Hkv, hd, causal, (Hq + 2 * Hkv) * hd};
    return st(spk_launch_attention((hipStream_t)stream, qkv, o, lse, a));
}

extern "C" int spk_kv_append(void* stream, const uint16_t* qkv, uint16_t* kt, uint16_t* v, int B, int S, int pos0,
                             int Hq, int Hkv, int hd, int max_len) {
    if (!qkv || !kt || !v || Hq < 1 || Hkv < 1 || hd < 1) return SP_ERR_INVALID_ARG;
    return st(spk_launch_kv_append((hipStream_t)stream, qkv, (Hq + 2 * Hkv) * hd, kt, v, B, S, pos0, Hq, Hkv, hd,
                                   max_len));
}

extern "C" int spk_decode_attention(void* stream, const uint16_t* qkv, const uint16_t* kt, const uint16_t* v,
                                    uint16_t* o, int B, int n, int max_len, int Hq, int Hkv, int hd) {
    if (!qkv || !kt || !v || !o || Hq < 1 || Hkv < 1) return SP_ERR_INVALID_ARG;
    return st(spk_launch_decode_attention((hipStream_t)stream, qkv, (Hq + 2 * Hkv) * hd, kt, v, o, Hq * hd, B, n,
                                          max_len, Hq, Hkv, hd));
}

extern "C" int spk_mse(void* stream, const float* y, const float* t, float* dy, uint16_t* dyb, float* scratch,
                       float* loss, size_t n) {
    if (!y || !t || !dy || !dyb || !scratch || !loss || n == 0) return SP_ERR_INVALID_ARG;
    return st(spk_launch_mse((hipStream_t)stream, y, t, dy, dyb, scratch, loss, n));
}

extern "C" int spk_swiglu_bwd(void* stream, const uint16_t* dz, uint16_t* gu, int T, int f) {
    if (!dz || !gu) return SP_ERR_INVALID_ARG;
    return st(spk_launch_swiglu_bwd((hipStream_t)stream, dz, gu, T, f));
}

extern "C" int spk_rmsnorm_bwd(void* stream, const float* da, const float* h, const uint16_t* gain, float* dh_io,
                               uint16_t* dhb, float* scratch, float* dgain, int T, int d, float eps) {
    if (!da || !h || !gain || !dh_io || !dhb || !scratch || !dgain) return SP_ERR_INVALID_ARG;
    return st(spk_launch_rmsnorm_bwd((hipStream_t)stream, da, h, gain, dh_io, dhb, scratch, dgain, T, d, eps));
}

static size_t al256(size_t v) { return (v + 255) / 256 * 256; }

extern "C" size_t spk_attention_bwd_scratch_bytes(int B, int S, int Hq, int Hkv, int hd) {
    if (B < 1 || S < 1 || Hq < 1 || Hkv < 1 || hd < 1) return 0;
    return al256((size_t)B * Hq * S * 4);     // delta = rowsum(dO * O)
}

extern "C" int spk_attention_bwd(void* stream, const uint16_t* qkv, const uint16_t* o, const uint16_t* dO,
                                 const float* lse, void* scratch, uint16_t* dqkv, int B, int S, int Hq, int Hkv,
                                 int hd, int causal) {
    if (!qkv || !o || !dO || !lse || !scratch || !dqkv || B < 1 || S < 1 || Hq < 1 || Hkv < 1) return SP_ERR_INVALID_ARG;
    if (hd != 64 && hd != 80 && hd != 128) return SP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    float* delta = static_cast<float*>(scratch);
    AttnShape a{B, S, Hq, Hkv, hd, causal, (Hq + 2 * Hkv) * hd};
    hipError_t e = spk_launch_attn_delta(s, dO, o, delta, B, S, Hq, hd);
    if (e != hipSuccess) return st(e);
    AttnBwdArgs g{qkv, dO, lse, delta, dqkv};
    return st(spk_launch_attention_bwd(s, g, a));
}

extern "C" int spk_layernorm_bwd(void* stream, const float* da, const float* h, const uint16_t* gain, float* dh_io,
                                 uint16_t* dhb, float* scratch, float* dgain, float* dbias, int T, int d, float eps) {
    if (!da || !h || !gain || !dh_io || !dhb || !scratch || !dgain || !dbias) return SP_ERR_INVALID_ARG;
    return st(spk_launch_layernorm_bwd((hipStream_t)stream, da, h, gain, dh_io, dhb, scratch, dgain, dbias, T, d, eps));
}

extern "C" int spk_gelu(void* stream, const uint16_t* u, uint16_t* z, size_t n) {
    if (!u || !z) return SP_ERR_INVALID_ARG;
    return st(spk_launch_gelu((hipStream_t)stream, u, z, n));
}

extern "C" int spk_gelu_bwd(void* stream, const uint16_t* dz, uint16_t* u, size_t n) {
    if (!dz || !u) return SP_ERR_INVALID_ARG;
    return st(spk_launch_gelu_bwd((hipStream_t)stream, dz, u, n));
}

extern "C" int spk_colsum_bf16(void* stream, const uint16_t* src, int ld, int T, int n, float* scratch, float* out) {
    if (!src || !scratch || !out) return SP_ERR_INVALID_ARG;
    return st(spk_launch_colsum_bf16((hipStream_t)stream, src, ld, T, n, scratch, out));
}
