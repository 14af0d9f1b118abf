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
    if (a_form < 0 || a_form > 1 || w_form < 0 || w_form > 1 || tile < 0 || tile > 3) return SP_ERR_INVALID_ARG;
    GemmArgs g{A, lda, a_form, W, ldw, w_form, C, ldc, R, ldr, bias, M, N, K, tile};
    return st(spk_launch_gemm((hipStream_t)stream, epilogue, g));
}

extern "C" int spk_swiglu(void* stream, const uint16_t* gu, uint16_t* z, int T, int f) {
    if (!gu || !z) return SP_ERR_INVALID_ARG;
    return st(spk_launch_swiglu((hipStream_t)stream, gu, z, T, f));
}

extern "C" size_t spk_attention_scratch_elems(int B, int S, int Hkv, int hd) {
    if (B < 1 || S < 1 || Hkv < 1 || hd < 1) return 0;
    return (size_t)B * Hkv * attn_hd_pad(hd) * attn_s_pad(S);
}

extern "C" int spk_attention(void* stream, const uint16_t* qkv, uint16_t* vt, uint16_t* o, float* lse, int B,
                             int S, int Hq, int Hkv, int hd, int causal) {
    if (!qkv || !vt || !o || B < 1 || S < 1 || Hq < 1 || Hkv < 1) return SP_ERR_INVALID_ARG;
    AttnShape a{B, S, Hq, Hkv, hd, causal, (Hq + 2 * Hkv) * hd};
    hipError_t e = spk_launch_transpose_v((hipStream_t)stream, qkv, vt, a);
    if (e != hipSuccess) return st(e);
    return st(spk_launch_attention((hipStream_t)stream, qkv, vt, o, lse, a));
}
