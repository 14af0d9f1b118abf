// Training step (paper Sec. 3.3: the window mechanism repeated for the backward
// pass).  Forward keeps every layer's fp32 input; the backward walks the layers
// in reverse, and when layer l's weights are back in a slot it recomputes the
// layer's internals from the saved input and runs the backward of every op.
// fp32 weight gradients are written into one of a few device gradient slots (same
// tensor order as the weight blob, offsets doubled) and streamed to the caller's
// pinned host blob on the device-to-host stream, fenced by one event pair per slot:
//   grad_ready[g]  compute -> d2h   (gradients of a layer complete)
//   gslot_free[g]  d2h -> compute   (slot g has been copied out, may be rewritten)
#include "sp_engine.h"

using namespace sp;

namespace {

struct LayerBufs {
    const float* h_in;   // layer input  fp32 [T,d]
    float* h_mid;        // after the attention residual
    float* h_out;        // layer output (nullptr: stop after the SwiGLU, recompute mode)
    float* lse;          // nullptr: not needed
};

// The activation set of a layer: the shared one, or the layer's own when activations are kept.
struct ActSet {
    bf16_t *a, *m, *qkv, *o, *gu, *z;
    float *h1, *lse;
};
ActSet act_set(sp_engine* e, int layer) {
    unsigned char* base = e->arena + (size_t)layer * e->ws.set_stride;
    auto P = [&](size_t off) { return base + off; };
    return ActSet{(bf16_t*)P(e->ws.a), (bf16_t*)P(e->ws.m), (bf16_t*)P(e->ws.qkv), (bf16_t*)P(e->ws.o),
                  (bf16_t*)P(e->ws.gu), (bf16_t*)P(e->ws.z), (float*)P(e->ws.h1), (float*)P(e->ws.lse)};
}

// Decoder layer with every intermediate kept in the activation set (a, qkv, o, m, gu, z).
int decoder_layer_keep(sp_engine* e, const unsigned char* w, const ActSet& as_, const LayerBufs& b, int B, int S) {
    const sp_stack_desc& d = e->desc;
    const Layout& L = e->lay;
    hipStream_t st = e->compute;
    const int T = B * S, dm = d.d_model, f = d.d_ffn;
    const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, nqkv = nq + 2 * nkv;
    auto W = [&](int t) { return reinterpret_cast<const bf16_t*>(w + L.t[t].offset); };
    bf16_t *a = as_.a, *m = as_.m, *qkv = as_.qkv, *o = as_.o, *gu = as_.gu, *z = as_.z;
    AttnShape as{B, S, d.n_q_heads, d.n_kv_heads, d.head_dim, d.causal, nqkv};
    GemmArgs g;
    SP_OP(e, SP_OP_NORM, spk_launch_norm(st, b.h_in, W(SP_T_G1), nullptr, a, T, dm, d.norm_eps));
    g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_WQKV), dm, OP_KMAJOR, qkv, nqkv, nullptr, 0, nullptr, T, nqkv, dm, 0};
    SP_OP(e, SP_OP_GEMM_QKV, spk_launch_gemm(st, EPI_BF16, g));
    SP_OP(e, SP_OP_ATTENTION, spk_launch_attention(st, qkv, o, b.lse, as));
    g = GemmArgs{o, nq, OP_KMAJOR, W(SP_T_WO), nq, OP_KMAJOR, b.h_mid, dm, b.h_in, dm, nullptr, T, dm, nq, 0};
    SP_OP(e, SP_OP_GEMM_O, spk_launch_gemm(st, EPI_RESID_F32, g));
    SP_OP(e, SP_OP_NORM, spk_launch_norm(st, b.h_mid, W(SP_T_G2), nullptr, m, T, dm, d.norm_eps));
    g = GemmArgs{m, dm, OP_KMAJOR, W(SP_T_WGU), dm, OP_KMAJOR, gu, 2 * f, nullptr, 0, nullptr, T, 2 * f, dm, 0};
    // every 4th launch of the largest GEMM is bracketed: the two event records cost a gap
    // on the stream, which on a compute-bound stack would show in the step time
    const bool kt = !e->kt_begin.empty() && (e->kt_seen++ % 4 == 0);
    const size_t kti = kt ? e->kt_count % e->kt_begin.size() : 0;
    if (kt) {
        SP_HIP(e, hipEventRecord(e->kt_begin[kti], st));
        e->kt_m = T; e->kt_n = 2 * f; e->kt_k = dm;
    }
    SP_OP(e, SP_OP_GEMM_FFN1, spk_launch_gemm(st, EPI_BF16, g));
    if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
    SP_OP(e, SP_OP_ACT, spk_launch_swiglu(st, gu, z, T, f));
    if (b.h_out) {
        g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_WD), f, OP_KMAJOR, b.h_out, dm, b.h_mid, dm, nullptr, T, dm, f, 0};
        SP_OP(e, SP_OP_GEMM_FFN2, spk_launch_gemm(st, EPI_RESID_F32, g));
    }
    return SP_OK;
}

// Encoder layer (pre-LayerNorm, biased linears, GELU) with every intermediate kept; the
// pre-activation u of the MLP goes where the decoder keeps [g | u], z = gelu(u) is a pass of
// its own because the backward needs both.
int encoder_layer_keep(sp_engine* e, const unsigned char* w, const ActSet& as_, const LayerBufs& b, int B, int S) {
    const sp_stack_desc& d = e->desc;
    const Layout& L = e->lay;
    hipStream_t st = e->compute;
    const int T = B * S, dm = d.d_model, f = d.d_ffn;
    const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, nqkv = nq + 2 * nkv;
    auto W = [&](int t) { return reinterpret_cast<const bf16_t*>(w + L.t[t].offset); };
    bf16_t *a = as_.a, *m = as_.m, *qkv = as_.qkv, *o = as_.o, *u = as_.gu, *z = as_.z;
    AttnShape as{B, S, d.n_q_heads, d.n_kv_heads, d.head_dim, d.causal, nqkv};
    GemmArgs g;
    SP_OP(e, SP_OP_NORM, spk_launch_norm(st, b.h_in, W(SP_T_LN1_G), W(SP_T_LN1_B), a, T, dm, d.norm_eps));
    g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_E_WQKV), dm, OP_KMAJOR, qkv, nqkv, nullptr, 0, W(SP_T_BQKV), T, nqkv, dm, 0};
    SP_OP(e, SP_OP_GEMM_QKV, spk_launch_gemm(st, EPI_BF16, g));
    SP_OP(e, SP_OP_ATTENTION, spk_launch_attention(st, qkv, o, b.lse, as));
    g = GemmArgs{o, nq, OP_KMAJOR, W(SP_T_E_WO), nq, OP_KMAJOR, b.h_mid, dm, b.h_in, dm, W(SP_T_BO), T, dm, nq, 0};
    SP_OP(e, SP_OP_GEMM_O, spk_launch_gemm(st, EPI_RESID_F32, g));
    SP_OP(e, SP_OP_NORM, spk_launch_norm(st, b.h_mid, W(SP_T_LN2_G), W(SP_T_LN2_B), m, T, dm, d.norm_eps));
    g = GemmArgs{m, dm, OP_KMAJOR, W(SP_T_W1), dm, OP_KMAJOR, u, f, nullptr, 0, W(SP_T_B1), T, f, dm, 0};
    const bool kt = !e->kt_begin.empty() && (e->kt_seen++ % 4 == 0);
    const size_t kti = kt ? e->kt_count % e->kt_begin.size() : 0;
    if (kt) {
        SP_HIP(e, hipEventRecord(e->kt_begin[kti], st));
        e->kt_m = T; e->kt_n = f; e->kt_k = dm;
    }
    SP_OP(e, SP_OP_GEMM_FFN1, spk_launch_gemm(st, EPI_BF16, g));
    if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
    SP_OP(e, SP_OP_ACT, spk_launch_gelu(st, u, z, (size_t)T * f));
    if (b.h_out) {
        g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_W2), f, OP_KMAJOR, b.h_out, dm, b.h_mid, dm, W(SP_T_B2), T, dm, f, 0};
        SP_OP(e, SP_OP_GEMM_FFN2, spk_launch_gemm(st, EPI_RESID_F32, g));
    }
    return SP_OK;
}

int layer_keep(sp_engine* e, const unsigned char* w, const ActSet& as_, const LayerBufs& b, int B, int S) {
    return e->desc.arch == SP_DECODER_SWIGLU_RMS ? decoder_layer_keep(e, w, as_, b, B, S)
                                                 : encoder_layer_keep(e, w, as_, b, B, S);
}

float* saved_input(sp_engine* e, int layer, int T) {
    return e->wsp<float>(e->ws.xs) + (size_t)layer * T * e->desc.d_model;
}

}  // namespace

int sp_train_begin(sp_engine* e, const float* x_dev, int B, int S) {
    const sp_stack_desc& d = e->desc;
    const int T = B * S;
    const int Tp = (T + 63) / 64 * 64;
    hipStream_t st = e->compute;
    if (Tp != T) {
        // token rows [T, Tp) of the buffers that feed the weight-gradient GEMMs (contraction
        // over tokens, padded to a multiple of 64) must read as zero
        const int nq = d.n_q_heads * d.head_dim, nqkv = nq + 2 * d.n_kv_heads * d.head_dim;
        struct { size_t off; int cols; bool per_set; } bufs[] = {
            {e->ws.a, d.d_model, true}, {e->ws.m, d.d_model, true}, {e->ws.o, nq, true},
            {e->ws.gu, (d.arch == SP_DECODER_SWIGLU_RMS ? 2 : 1) * d.d_ffn, true}, {e->ws.z, d.d_ffn, true},
            {e->ws.dhb, d.d_model, false}, {e->ws.dqkv, nqkv, false}};
        const int n_sets = e->ws.set_stride ? d.n_layers : 1;
        for (auto& bf : bufs)
            for (int set = 0; set < (bf.per_set ? n_sets : 1); ++set) {
                uint32_t* p = reinterpret_cast<uint32_t*>(e->arena + (size_t)set * e->ws.set_stride + bf.off +
                                                          (size_t)T * bf.cols * 2);
                SP_OP(e, SP_OP_COPY, spk_launch_fill_u32(st, p, 0u, (size_t)(Tp - T) * bf.cols / 2));
            }
    }
    SP_OP(e, SP_OP_COPY, spk_launch_copy_f32(st, x_dev, saved_input(e, 0, T), (size_t)T * d.d_model));
    return SP_OK;
}

int sp_layer_forward_train(sp_engine* e, int layer, const unsigned char* w, int B, int S) {
    const int T = B * S, L = e->desc.n_layers;
    // the last layer writes y (the caller's buffer, or the stream-gradient buffer that the
    // loss kernel then turns into dy in place)
    float* out = layer + 1 < L ? saved_input(e, layer + 1, T) : (e->y_out ? e->y_out : e->wsp<float>(e->ws.dh));
    const ActSet as_ = act_set(e, layer);
    // with kept activations the forward also produces what the backward needs (log-sum-exp)
    LayerBufs b{saved_input(e, layer, T), as_.h1, out, e->ws.set_stride ? as_.lse : nullptr};
    return layer_keep(e, w, as_, b, B, S);
}

int sp_train_loss(sp_engine* e, const float* target_dev, float* loss_dev, int B, int S) {
    const size_t n = (size_t)B * S * e->desc.d_model;
    float* dh = e->wsp<float>(e->ws.dh);
    const float* y = e->y_out ? e->y_out : dh;
    SP_OP(e, SP_OP_LOSS, spk_launch_mse(e->compute, y, target_dev, dh, e->wsp<bf16_t>(e->ws.dhb), e->wsp<float>(e->ws.part),
                                        loss_dev, n));
    return SP_OK;
}

int sp_layer_backward(sp_engine* e, int layer, const unsigned char* w, int B, int S) {
    const sp_stack_desc& d = e->desc;
    const Layout& L = e->lay;
    hipStream_t st = e->compute;
    const int T = B * S, Tp = (T + 63) / 64 * 64, dm = d.d_model, f = d.d_ffn;
    const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, nqkv = nq + 2 * nkv;
    auto W = [&](int t) { return reinterpret_cast<const bf16_t*>(w + L.t[t].offset); };
    // a frozen layer only passes the gradient on to its input: no weight-gradient GEMMs, no
    // copy to the host (its gain gradients land in the slot and are dropped)
    const bool frozen = layer < e->frozen;
    const int gs = e->gslot_next;
    e->gslot_next = (gs + 1) % sp::kGradSlots;
    unsigned char* gslot = e->arena + e->ws.gslot[gs];
    auto G = [&](int t) { return reinterpret_cast<float*>(gslot + 2 * L.t[t].offset); };
    if (e->gslot_used[gs]) SP_HIP(e, hipStreamWaitEvent(st, e->gslot_free[gs], 0));

    const ActSet as_ = act_set(e, layer);
    float* x_l = saved_input(e, layer, T);
    float* h1 = as_.h1;
    float* lse = as_.lse;
    float* delta = e->wsp<float>(e->ws.delta);
    float* dh = e->wsp<float>(e->ws.dh);
    float* da = e->wsp<float>(e->ws.da);
    float* part = e->wsp<float>(e->ws.part);
    bf16_t *a = as_.a, *m = as_.m, *qkv = as_.qkv, *o = as_.o, *gu = as_.gu, *z = as_.z;
    bf16_t* dhb = e->wsp<bf16_t>(e->ws.dhb);
    bf16_t* dz = e->wsp<bf16_t>(e->ws.dz);
    bf16_t* dob = e->wsp<bf16_t>(e->ws.dob);
    bf16_t* dqkv = e->wsp<bf16_t>(e->ws.dqkv);
    AttnShape as{B, S, d.n_q_heads, d.n_kv_heads, d.head_dim, d.causal, nqkv};
    GemmArgs g;

    // recompute a, qkv, o, lse, h1, m, gu, z from the saved input -- unless the forward kept them
    if (!e->ws.set_stride) {
        LayerBufs lb{x_l, h1, nullptr, lse};
        int rc = layer_keep(e, w, as_, lb, B, S);
        if (rc != SP_OK) return rc;
    }

    const bool dec = d.arch == SP_DECODER_SWIGLU_RMS;
    const int t_wo = dec ? SP_T_WO : SP_T_E_WO, t_wqkv = dec ? SP_T_WQKV : SP_T_E_WQKV;
    // bias gradient of a linear map = column sums of its output gradient over the tokens
    auto bias_grad = [&](const bf16_t* dy, int n, int t) -> int {
        if (frozen) return SP_OK;
        SP_OP(e, SP_OP_BIAS_GRAD, spk_launch_colsum_bf16(st, dy, n, T, n, part, G(t)));
        return SP_OK;
    };
    int rc;

    // ---- FFN.  dh is dL/d(layer output); dhb its bf16 copy.
    if (dec) {
        // dWd[d,f] = dh^T z       (contraction over tokens: both operands transposed on the way in)
        g = GemmArgs{dhb, dm, OP_RMAJOR, z, f, OP_RMAJOR, G(SP_T_WD), f, nullptr, 0, nullptr, dm, f, Tp, 0};
        if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
        // dz[T,f] = dh Wd         (Wd is [d,f]: its row index f is contiguous)
        g = GemmArgs{dhb, dm, OP_KMAJOR, W(SP_T_WD), f, OP_RMAJOR, dz, f, nullptr, 0, nullptr, T, f, dm, 0};
        SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_BF16, g));
        // [dg | du] in place over [g | u]
        SP_OP(e, SP_OP_ACT_BWD, spk_launch_swiglu_bwd(st, dz, gu, T, f));
        // dWgu[2f,d] = dgu^T m
        g = GemmArgs{gu, 2 * f, OP_RMAJOR, m, dm, OP_RMAJOR, G(SP_T_WGU), dm, nullptr, 0, nullptr, 2 * f, dm, Tp, 0};
        if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
        // dm[T,d] = dgu Wgu  (fp32)
        g = GemmArgs{gu, 2 * f, OP_KMAJOR, W(SP_T_WGU), dm, OP_RMAJOR, da, dm, nullptr, 0, nullptr, T, dm, 2 * f, 0};
        SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_F32, g));
        // second norm: dh += d(rmsnorm)(h1) applied to dm; dg2
        SP_OP(e, SP_OP_NORM_BWD, spk_launch_rmsnorm_bwd(st, da, h1, W(SP_T_G2), dh, dhb, part, G(SP_T_G2), T, dm, d.norm_eps));
    } else {
        bf16_t* u = gu;                     // pre-activation of the MLP, [T, f]
        if ((rc = bias_grad(dhb, dm, SP_T_B2)) != SP_OK) return rc;
        // dW2[d,f] = dh^T z
        g = GemmArgs{dhb, dm, OP_RMAJOR, z, f, OP_RMAJOR, G(SP_T_W2), f, nullptr, 0, nullptr, dm, f, Tp, 0};
        if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
        // dz[T,f] = dh W2
        g = GemmArgs{dhb, dm, OP_KMAJOR, W(SP_T_W2), f, OP_RMAJOR, dz, f, nullptr, 0, nullptr, T, f, dm, 0};
        SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_BF16, g));
        // du = dz gelu'(u), in place over u
        SP_OP(e, SP_OP_ACT_BWD, spk_launch_gelu_bwd(st, dz, u, (size_t)T * f));
        if ((rc = bias_grad(u, f, SP_T_B1)) != SP_OK) return rc;
        // dW1[f,d] = du^T m
        g = GemmArgs{u, f, OP_RMAJOR, m, dm, OP_RMAJOR, G(SP_T_W1), dm, nullptr, 0, nullptr, f, dm, Tp, 0};
        if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
        // dm[T,d] = du W1  (fp32)
        g = GemmArgs{u, f, OP_KMAJOR, W(SP_T_W1), dm, OP_RMAJOR, da, dm, nullptr, 0, nullptr, T, dm, f, 0};
        SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_F32, g));
        // second norm: dh += d(layernorm)(h1) applied to dm; its gain and bias gradients
        SP_OP(e, SP_OP_NORM_BWD, spk_launch_layernorm_bwd(st, da, h1, W(SP_T_LN2_G), dh, dhb, part, G(SP_T_LN2_G), G(SP_T_LN2_B), T,
                                           dm, d.norm_eps));
    }

    // ---- attention block.  dh is now dL/dh1.
    if (!dec && (rc = bias_grad(dhb, dm, SP_T_BO)) != SP_OK) return rc;
    // dWo[d,nq] = dh^T o
    g = GemmArgs{dhb, dm, OP_RMAJOR, o, nq, OP_RMAJOR, G(t_wo), nq, nullptr, 0, nullptr, dm, nq, Tp, 0};
    if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
    // do[T,nq] = dh Wo
    g = GemmArgs{dhb, dm, OP_KMAJOR, W(t_wo), nq, OP_RMAJOR, dob, nq, nullptr, 0, nullptr, T, nq, dm, 0};
    SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_BF16, g));
    SP_OP(e, SP_OP_ATTENTION_BWD, spk_launch_attn_delta(st, dob, o, delta, B, S, d.n_q_heads, d.head_dim));
    AttnBwdArgs ab{qkv, dob, lse, delta, dqkv};
    SP_OP(e, SP_OP_ATTENTION_BWD, spk_launch_attention_bwd(st, ab, as));
    if (!dec && (rc = bias_grad(dqkv, nqkv, SP_T_BQKV)) != SP_OK) return rc;
    // dWqkv[nqkv,d] = dqkv^T a
    g = GemmArgs{dqkv, nqkv, OP_RMAJOR, a, dm, OP_RMAJOR, G(t_wqkv), dm, nullptr, 0, nullptr, nqkv, dm, Tp, 0};
    if (!frozen) SP_OP(e, SP_OP_GEMM_DW, spk_launch_gemm(st, EPI_F32, g));
    // da[T,d] = dqkv Wqkv (fp32)
    g = GemmArgs{dqkv, nqkv, OP_KMAJOR, W(t_wqkv), dm, OP_RMAJOR, da, dm, nullptr, 0, nullptr, T, dm, nqkv, 0};
    SP_OP(e, SP_OP_GEMM_DX, spk_launch_gemm(st, EPI_F32, g));
    // first norm: dh += d(norm)(x_l) applied to da; its parameter gradients.  dh is now
    // dL/d(layer input).
    if (dec)
        SP_OP(e, SP_OP_NORM_BWD, spk_launch_rmsnorm_bwd(st, da, x_l, W(SP_T_G1), dh, dhb, part, G(SP_T_G1), T, dm, d.norm_eps));
    else
        SP_OP(e, SP_OP_NORM_BWD, spk_launch_layernorm_bwd(st, da, x_l, W(SP_T_LN1_G), dh, dhb, part, G(SP_T_LN1_G), G(SP_T_LN1_B), T,
                                           dm, d.norm_eps));

    if (frozen) return SP_OK;
    // ---- hand the gradient slot to the device-to-host stream
    SP_HIP(e, hipEventRecord(e->grad_ready[gs], st));
    SP_HIP(e, hipStreamWaitEvent(e->d2h, e->grad_ready[gs], 0));
    SP_HIP(e, hipMemcpyAsync(e->grad_blobs[layer], gslot, L.grad_bytes, hipMemcpyDeviceToHost, e->d2h));
    SP_HIP(e, hipEventRecord(e->gslot_free[gs], e->d2h));
    SP_HIP(e, hipEventRecord(e->grad_landed[layer], e->d2h));
    e->grad_sent[layer] = 1;
    e->last_grad_copy = e->gslot_free[gs];
    e->gslot_used[gs] = 1;
    e->stats_d2h_copies++;
    e->stats_d2h_bytes += L.grad_bytes;
    return SP_OK;
}

int sp_train_end(sp_engine* e, float* dx_dev, int B, int S) {
    if (dx_dev)
        SP_OP(e, SP_OP_COPY, spk_launch_copy_f32(e->compute, e->wsp<float>(e->ws.dh), dx_dev, (size_t)B * S * e->desc.d_model));
    return SP_OK;
}
