// The transfer engine and per-layer executor behind sp_create / sp_forward /
// sp_forward_backward / sp_destroy.
//
// HBM holds n_slots layer-sized slots carved from the caller's arena.  The
// scheduler (sp_host.hip) decides which layer goes to which slot; this file
// turns each decision into stream work:
//   copy(l -> slot):  h2d stream waits done[prev user of slot]; one
//                     hipMemcpyAsync of the whole layer blob; record loaded[l]
//   compute(l):       compute stream waits loaded[l]; the layer's kernels;
//                     record done[l]
// Those two event kinds are the only cross-stream edges.  An event is always
// recorded (in host order) before anything waits on it.  Nothing here blocks
// the host, and no device memory is allocated.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <set>
#include <string>
#include <vector>

#include "sp_engine.h"

using namespace sp;

namespace {
thread_local std::string g_create_error;
std::mutex g_live_mu;
std::set<sp_engine*> g_live;   // handles between sp_create and sp_destroy

bool is_live(sp_engine* e) {
    std::lock_guard<std::mutex> lk(g_live_mu);
    return g_live.count(e) != 0;
}
}  // namespace

int sp_fail(sp_engine* e, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (e) e->error = buf; else g_create_error = buf;
    return code;
}
#define fail sp_fail

// ---- the sink that enqueues real stream work -------------------------------------
struct HipSink : SchedSink {
    sp_engine* e;
    float* hbuf;        // forward: the residual stream (fp32 [T, d]) being updated in place
    int B, S;
    bool training_fwd = false;
    explicit HipSink(sp_engine* eng) : e(eng), hbuf(nullptr), B(0), S(0) {}

    int copy(int layer, int slot, int wait_layer) override {
        hipStream_t cs = e->h2d;
        if (e->flags & SP_FLAG_NO_OVERLAP) {
            // Naive comparator: a copy starts only after everything enqueued for compute.
            SP_HIP(e, hipEventRecord(e->ev_sync_c, e->compute));
            SP_HIP(e, hipStreamWaitEvent(cs, e->ev_sync_c, 0));
        } else if (wait_layer >= 0 && e->done_recorded[wait_layer]) {
            SP_HIP(e, hipStreamWaitEvent(cs, e->done[wait_layer], 0));
        }
        unsigned char* dst = e->slots + (size_t)slot * e->plan.slot_bytes;
        if (e->flags & SP_FLAG_POISON) {
            // bf16 NaN pattern: a read of a slot before its copy lands shows up as NaN output
            SP_HIP(e, spk_launch_fill_u32(cs, reinterpret_cast<uint32_t*>(dst), 0x7FC17FC1u, e->plan.slot_bytes / 4));
        }
        const bool timed = (e->flags & SP_FLAG_TIMING) && e->copy_n < SP_MAX_TRACE_LAYERS;
        if (timed) SP_HIP(e, hipEventRecord(e->t_copy_begin[e->copy_n], cs));
        SP_HIP(e, hipMemcpyAsync(dst, e->blobs[layer], e->lay.blob_bytes, hipMemcpyHostToDevice, cs));
        if (timed) {
            SP_HIP(e, hipEventRecord(e->t_copy_end[e->copy_n], cs));
            e->copy_layer[e->copy_n++] = layer;
        }
        SP_HIP(e, hipEventRecord(e->loaded[layer], cs));
        e->loaded_recorded[layer] = 1;
        e->stats_h2d_copies++;
        e->stats_h2d_bytes += e->lay.blob_bytes;
        e->call_h2d_copies++;
        e->call_h2d_bytes += e->lay.blob_bytes;
        return SP_OK;
    }

    int compute(int layer, int slot, int dir, bool /*fresh*/) override {
        hipStream_t st = e->compute;
        if (e->flags & SP_FLAG_NO_OVERLAP) {
            // Naive comparator: compute starts only after every copy enqueued so far.
            SP_HIP(e, hipEventRecord(e->ev_sync_h, e->h2d));
            SP_HIP(e, hipStreamWaitEvent(st, e->ev_sync_h, 0));
        } else if (e->loaded_recorded[layer]) {
            SP_HIP(e, hipStreamWaitEvent(st, e->loaded[layer], 0));
        }
        const unsigned char* w = e->slots + (size_t)slot * e->plan.slot_bytes;
        const bool timed = (e->flags & SP_FLAG_TIMING) && e->trace_n < SP_MAX_TRACE_LAYERS;
        if (timed) SP_HIP(e, hipEventRecord(e->t_comp_begin[e->trace_n], st));
        int rc;
        if (dir > 0)
            rc = training_fwd ? sp_layer_forward_train(e, layer, w, B, S) : sp_layer_forward(e, w, hbuf, B, S);
        else
            rc = sp_layer_backward(e, layer, w, B, S);
        if (rc != SP_OK) return rc;
        if (timed) {
            SP_HIP(e, hipEventRecord(e->t_comp_end[e->trace_n], st));
            e->trace_layer[e->trace_n] = layer;
            e->trace_n++;
        }
        SP_HIP(e, hipEventRecord(e->done[layer], st));
        e->done_recorded[layer] = 1;
        return SP_OK;
    }
};

// ---- one decoder / encoder layer, forward, residual stream updated in place -------
int sp_layer_forward(sp_engine* e, const unsigned char* w, float* h, int B, int S) {
    const sp_stack_desc& d = e->desc;
    const Layout& L = e->lay;
    hipStream_t st = e->compute;
    const int T = B * S, dm = d.d_model, f = d.d_ffn;
    const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, nqkv = nq + 2 * nkv;
    auto W = [&](int t) { return reinterpret_cast<const bf16_t*>(w + L.t[t].offset); };
    bf16_t* a = e->wsp<bf16_t>(e->ws.a);
    bf16_t* qkv = e->wsp<bf16_t>(e->ws.qkv);
    bf16_t* vt = e->wsp<bf16_t>(e->ws.vt);
    bf16_t* o = e->wsp<bf16_t>(e->ws.o);
    bf16_t* gu = e->wsp<bf16_t>(e->ws.gu);
    bf16_t* z = e->wsp<bf16_t>(e->ws.z);
    const bool dec = d.arch == SP_DECODER_SWIGLU_RMS;
    AttnShape as{B, S, d.n_q_heads, d.n_kv_heads, d.head_dim, d.causal, nqkv};
    GemmArgs g;

    // b1: a = norm(h)
    SP_HIP(e, spk_launch_norm(st, h, W(dec ? SP_T_G1 : SP_T_LN1_G), dec ? nullptr : W(SP_T_LN1_B), a, T, dm, d.norm_eps));
    // b2: qkv = a Wqkv^T (+ b)
    g = GemmArgs{a, dm, OP_KMAJOR, W(dec ? SP_T_WQKV : SP_T_E_WQKV), dm, OP_KMAJOR, qkv, nqkv, nullptr, 0,
                 dec ? nullptr : W(SP_T_BQKV), T, nqkv, dm, e->gemm_tile};
    SP_HIP(e, spk_launch_gemm(st, EPI_BF16, g));
    // b3: attention
    SP_HIP(e, spk_launch_transpose_v(st, qkv, vt, as));
    SP_HIP(e, spk_launch_attention(st, qkv, vt, o, nullptr, as));
    // b4: h += o Wo^T (+ b)
    g = GemmArgs{o, nq, OP_KMAJOR, W(dec ? SP_T_WO : SP_T_E_WO), nq, OP_KMAJOR, h, dm, h, dm,
                 dec ? nullptr : W(SP_T_BO), T, dm, nq, e->gemm_tile};
    SP_HIP(e, spk_launch_gemm(st, EPI_RESID_F32, g));
    // b5: a = norm(h)
    SP_HIP(e, spk_launch_norm(st, h, W(dec ? SP_T_G2 : SP_T_LN2_G), dec ? nullptr : W(SP_T_LN2_B), a, T, dm, d.norm_eps));
    const bool kt = (e->flags & SP_FLAG_TIMING) && !e->kt_begin.empty();
    const size_t kti = kt ? e->kt_count % e->kt_begin.size() : 0;
    if (kt) {
        SP_HIP(e, hipEventRecord(e->kt_begin[kti], st));
        e->kt_m = T; e->kt_n = dec ? 2 * f : f; e->kt_k = dm;
    }
    if (dec) {
        // b6+b7: z = silu(a Wg^T) * (a Wu^T), gate applied in the GEMM epilogue
        if (e->fuse_swiglu) {
            g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_WGU), dm, OP_KMAJOR, z, f, nullptr, 0, nullptr, T, f, dm, e->gemm_tile};
            SP_HIP(e, spk_launch_gemm(st, EPI_SWIGLU_BF16, g));
        } else {
            g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_WGU), dm, OP_KMAJOR, gu, 2 * f, nullptr, 0, nullptr, T, 2 * f, dm, e->gemm_tile};
            SP_HIP(e, spk_launch_gemm(st, EPI_BF16, g));
        }
        if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
        if (!e->fuse_swiglu) SP_HIP(e, spk_launch_swiglu(st, gu, z, T, f));
        // b8: h += z Wd^T
        g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_WD), f, OP_KMAJOR, h, dm, h, dm, nullptr, T, dm, f, e->gemm_tile};
        SP_HIP(e, spk_launch_gemm(st, EPI_RESID_F32, g));
    } else {
        g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_W1), dm, OP_KMAJOR, z, f, nullptr, 0, W(SP_T_B1), T, f, dm, e->gemm_tile};
        SP_HIP(e, spk_launch_gemm(st, EPI_GELU_BF16, g));
        if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
        g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_W2), f, OP_KMAJOR, h, dm, h, dm, W(SP_T_B2), T, dm, f, e->gemm_tile};
        SP_HIP(e, spk_launch_gemm(st, EPI_RESID_F32, g));
    }
    return SP_OK;
}

// ---- C entry points -------------------------------------------------------------------
static int destroy_engine(sp_engine* e);

extern "C" const char* sp_last_error(sp_handle h) { return (h && is_live(h)) ? h->error.c_str() : g_create_error.c_str(); }

extern "C" int sp_create(sp_handle* out, const sp_stack_desc* desc, const void* const* blobs, const sp_config* cfg) {
    if (!out) return fail(nullptr, SP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    const char* why = nullptr;
    if (validate_desc(desc, &why) != SP_OK) return fail(nullptr, SP_ERR_INVALID_ARG, "bad stack desc: %s", why);
    if (!cfg || cfg->struct_size != sizeof(sp_config)) return fail(nullptr, SP_ERR_INVALID_ARG, "bad config struct");
    if (!blobs) return fail(nullptr, SP_ERR_INVALID_ARG, "layer_host_blobs is NULL");
    if (cfg->resident_window_k < 1 || cfg->prefetch_depth_p < 1) return fail(nullptr, SP_ERR_INVALID_ARG, "k and p must be >= 1");
    if (!cfg->device_arena || ((uintptr_t)cfg->device_arena & (kSlotAlign - 1)))
        return fail(nullptr, SP_ERR_INVALID_ARG, "device_arena must be non-NULL and 4 KiB aligned");
    const bool training = cfg->flags & SP_FLAG_TRAINING;
    if (cfg->h2d_stream == cfg->compute_stream) return fail(nullptr, SP_ERR_INVALID_ARG, "h2d_stream must differ from compute_stream");
    if (training && (!cfg->d2h_stream || cfg->d2h_stream == cfg->compute_stream || cfg->d2h_stream == cfg->h2d_stream))
        return fail(nullptr, SP_ERR_INVALID_ARG, "training needs a d2h_stream distinct from the other two");
    if (training && desc->arch != SP_DECODER_SWIGLU_RMS)
        return fail(nullptr, SP_ERR_INVALID_ARG, "training is implemented for decoder stacks only");
    if (desc->n_layers > 4096) return fail(nullptr, SP_ERR_INVALID_ARG, "n_layers > 4096");
    sp_plan plan;
    int rc = make_plan(desc, cfg->resident_window_k, cfg->prefetch_depth_p, cfg->gpu_budget_bytes, training, &plan);
    if (rc == SP_ERR_BUDGET) {
        return fail(nullptr, rc, "gpu_budget_bytes=%llu cannot hold the workspace (%llu) plus one layer slot (%llu)",
                    (unsigned long long)cfg->gpu_budget_bytes, (unsigned long long)plan.workspace_bytes,
                    (unsigned long long)plan.slot_bytes);
    }
    if (rc != SP_OK) return fail(nullptr, rc, "cannot plan");
    for (int l = 0; l < desc->n_layers; ++l) {
        if (!blobs[l]) return fail(nullptr, SP_ERR_INVALID_ARG, "layer_host_blobs[%d] is NULL", l);
        hipPointerAttribute_t at;
        hipError_t pe = hipPointerGetAttributes(&at, blobs[l]);
        if (pe != hipSuccess || at.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            return fail(nullptr, SP_ERR_NOT_PINNED, "layer_host_blobs[%d] is not pinned host memory", l);
        }
    }
    sp_engine* e = new (std::nothrow) sp_engine();
    if (!e) return fail(nullptr, SP_ERR_INVALID_ARG, "out of host memory");
    e->desc = *desc;
    e->flags = cfg->flags;
    e->plan = plan;
    make_layout(desc, &e->lay);
    make_workspace(desc, e->lay, training, &e->ws);
    e->arena = static_cast<unsigned char*>(cfg->device_arena);
    e->slots = e->arena + e->ws.total;
    e->compute = static_cast<hipStream_t>(cfg->compute_stream);
    e->h2d = static_cast<hipStream_t>(cfg->h2d_stream);
    e->d2h = static_cast<hipStream_t>(cfg->d2h_stream);
    e->blobs.assign(blobs, blobs + desc->n_layers);
    const int L = desc->n_layers;
    e->loaded.assign(L, nullptr);
    e->done.assign(L, nullptr);
    e->loaded_recorded.assign(L, 0);
    e->done_recorded.assign(L, 0);
    const unsigned evflags = (cfg->flags & SP_FLAG_TIMING) ? hipEventDefault : hipEventDisableTiming;
    auto mk = [&](hipEvent_t* ev, unsigned fl) { return hipEventCreateWithFlags(ev, fl); };
    hipError_t he = hipSuccess;
    for (int l = 0; l < L && he == hipSuccess; ++l) {
        he = mk(&e->loaded[l], evflags);
        if (he == hipSuccess) he = mk(&e->done[l], evflags);
    }
    if (he == hipSuccess) he = mk(&e->ev_sync_c, hipEventDisableTiming);
    if (he == hipSuccess) he = mk(&e->ev_sync_h, hipEventDisableTiming);
    for (int i = 0; i < 2 && he == hipSuccess; ++i) {
        he = mk(&e->grad_ready[i], hipEventDisableTiming);
        if (he == hipSuccess) he = mk(&e->gslot_free[i], hipEventDisableTiming);
    }
    if (he == hipSuccess && (cfg->flags & SP_FLAG_TIMING)) {
        he = mk(&e->t0, hipEventDefault);
        for (int i = 0; i < SP_MAX_TRACE_LAYERS && he == hipSuccess; ++i) {
            he = mk(&e->t_copy_begin[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->t_copy_end[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->t_comp_begin[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->t_comp_end[i], hipEventDefault);
        }
    }
    if (he == hipSuccess && (cfg->flags & SP_FLAG_TIMING)) {
        e->kt_begin.assign(2048, nullptr);
        e->kt_end.assign(2048, nullptr);
        for (size_t i = 0; i < e->kt_begin.size() && he == hipSuccess; ++i) {
            he = mk(&e->kt_begin[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->kt_end[i], hipEventDefault);
        }
    }
    if (he != hipSuccess) {
        fail(nullptr, SP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(he));
        destroy_engine(e);
        return SP_ERR_HIP;
    }
    const bool naive = cfg->flags & SP_FLAG_NO_OVERLAP;
    e->sched.reset(L, plan.n_slots, naive ? plan.n_slots : plan.p_eff);
    e->fuse_swiglu = !training;
    e->gemm_tile = 0;
    if (const char* t = getenv("SP_GEMM_TILE")) e->gemm_tile = atoi(t);
    if (const char* t = getenv("SP_FUSE_SWIGLU")) e->fuse_swiglu = atoi(t) != 0 && !training;
    if (training) {
        // padded token rows of the GEMM-operand buffers must read as zero
        hipError_t fe = spk_launch_fill_u32(e->compute, reinterpret_cast<uint32_t*>(e->arena), 0u, e->ws.total / 4);
        if (fe != hipSuccess) {
            fail(nullptr, SP_ERR_HIP, "workspace clear failed: %s", hipGetErrorString(fe));
            destroy_engine(e);
            return SP_ERR_HIP;
        }
    }
    {
        std::lock_guard<std::mutex> lk(g_live_mu);
        g_live.insert(e);
    }
    *out = e;
    return SP_OK;
}

static int check_call(sp_engine* e, int B, int S) {
    if (!e) return SP_ERR_INVALID_ARG;
    if (!is_live(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (destroyed or never created)");
    if (B < 1 || S < 1 || B > e->desc.max_batch || S > e->desc.max_seq)
        return fail(e, SP_ERR_SHAPE, "B=%d S=%d outside 1..%d x 1..%d", B, S, e->desc.max_batch, e->desc.max_seq);
    return SP_OK;
}

static int begin_call(sp_engine* e) {
    e->call_h2d_copies = e->call_h2d_bytes = 0;
    e->trace_n = 0;
    e->copy_n = 0;
    if (e->flags & SP_FLAG_TIMING) SP_HIP(e, hipEventRecord(e->t0, e->compute));
    return SP_OK;
}

extern "C" int sp_forward(sp_handle e, const float* x_dev, float* y_dev, int B, int S) {
    int rc = check_call(e, B, S);
    if (rc != SP_OK) return rc;
    if (!x_dev || !y_dev) return fail(e, SP_ERR_INVALID_ARG, "x_dev / y_dev is NULL");
    if (((uintptr_t)x_dev | (uintptr_t)y_dev) & 15) return fail(e, SP_ERR_INVALID_ARG, "x_dev / y_dev must be 16-byte aligned");
    if ((rc = begin_call(e)) != SP_OK) return rc;
    SP_HIP(e, spk_launch_copy_f32(e->compute, x_dev, y_dev, (size_t)B * S * e->desc.d_model));
    HipSink sink(e);
    sink.hbuf = y_dev;
    sink.B = B;
    sink.S = S;
    const bool wrap = (e->flags & SP_FLAG_WRAP_PREFETCH) && !(e->flags & SP_FLAG_TRAINING);
    rc = e->sched.run_pass(+1, wrap, sink);
    if (rc != SP_OK) return rc;
    e->calls++;
    return SP_OK;
}

extern "C" int sp_get_stats(sp_handle e, sp_stats* out) {
    if (!e || !out) return SP_ERR_INVALID_ARG;
    if (!is_live(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (destroyed or never created)");
    memset(out, 0, sizeof(*out));
    out->struct_size = sizeof(sp_stats);
    out->plan = e->plan;
    out->calls = e->calls;
    out->h2d_copies = e->stats_h2d_copies;
    out->h2d_bytes = e->stats_h2d_bytes;
    out->d2h_copies = e->stats_d2h_copies;
    out->d2h_bytes = e->stats_d2h_bytes;
    out->last_h2d_copies = e->call_h2d_copies;
    out->last_h2d_bytes = e->call_h2d_bytes;
    if (!(e->flags & SP_FLAG_TIMING) || e->calls == 0) return SP_OK;
    SP_HIP(e, hipStreamSynchronize(e->h2d));
    SP_HIP(e, hipStreamSynchronize(e->compute));
    if (e->d2h) SP_HIP(e, hipStreamSynchronize(e->d2h));
    {
        const uint32_t cnt = (uint32_t)std::min<size_t>(e->kt_count, e->kt_begin.size());
        for (uint32_t i = 0; i < cnt; ++i) {
            float ms = 0;
            SP_HIP(e, hipEventElapsedTime(&ms, e->kt_begin[i], e->kt_end[i]));
            out->big_gemm_ms_sum += ms;
        }
        out->big_gemm_launches = cnt;
        out->big_gemm_m = e->kt_m; out->big_gemm_n = e->kt_n; out->big_gemm_k = e->kt_k;
        e->kt_count = 0;
    }
    const int n = e->trace_n;
    out->n_timed = n;
    std::vector<std::pair<float, float>> comp(n);
    float tmin = 1e30f, tmax = -1e30f;
    for (int i = 0; i < n; ++i) {
        float b = 0, en = 0;
        SP_HIP(e, hipEventElapsedTime(&b, e->t0, e->t_comp_begin[i]));
        SP_HIP(e, hipEventElapsedTime(&en, e->t0, e->t_comp_end[i]));
        out->comp_begin_ms[i] = b;
        out->comp_end_ms[i] = en;
        out->copy_begin_ms[i] = out->copy_end_ms[i] = -1.f;
        comp[i] = {b, en};
        out->compute_busy_ms += en - b;
        tmin = std::min(tmin, b);
        tmax = std::max(tmax, en);
    }
    std::sort(comp.begin(), comp.end());
    const int nc = e->copy_n;
    for (int c = 0; c < nc; ++c) {
        float b = 0, en = 0;
        SP_HIP(e, hipEventElapsedTime(&b, e->t0, e->t_copy_begin[c]));
        SP_HIP(e, hipEventElapsedTime(&en, e->t0, e->t_copy_end[c]));
        // attach to the first traced compute of that layer (reporting only)
        for (int i = 0; i < n; ++i)
            if (e->trace_layer[i] == e->copy_layer[c] && out->copy_begin_ms[i] < 0.f && out->comp_begin_ms[i] >= b) {
                out->copy_begin_ms[i] = b;
                out->copy_end_ms[i] = en;
                break;
            }
        out->copy_busy_ms += en - b;
        for (auto& iv : comp) {
            const float lo = std::max(b, iv.first), hi = std::min(en, iv.second);
            if (hi > lo) out->copy_hidden_ms += hi - lo;
        }
        tmin = std::min(tmin, b);
        tmax = std::max(tmax, en);
    }
    out->wall_ms = (n || nc) ? tmax - tmin : 0.f;
    return SP_OK;
}

extern "C" int sp_destroy(sp_handle e) {
    if (!e) return SP_ERR_INVALID_ARG;
    {
        std::lock_guard<std::mutex> lk(g_live_mu);
        if (!g_live.erase(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (double destroy?)");
    }
    return destroy_engine(e);
}

static int destroy_engine(sp_engine* e) {
    if (e->h2d) (void)hipStreamSynchronize(e->h2d);
    (void)hipStreamSynchronize(e->compute);
    if (e->d2h) (void)hipStreamSynchronize(e->d2h);
    auto kill = [](hipEvent_t ev) { if (ev) (void)hipEventDestroy(ev); };
    for (auto ev : e->loaded) kill(ev);
    for (auto ev : e->done) kill(ev);
    kill(e->ev_sync_c);
    kill(e->ev_sync_h);
    kill(e->t0);
    for (int i = 0; i < 2; ++i) { kill(e->grad_ready[i]); kill(e->gslot_free[i]); }
    for (auto ev : e->kt_begin) kill(ev);
    for (auto ev : e->kt_end) kill(ev);
    for (int i = 0; i < SP_MAX_TRACE_LAYERS; ++i) {
        kill(e->t_copy_begin[i]); kill(e->t_copy_end[i]); kill(e->t_comp_begin[i]); kill(e->t_comp_end[i]);
    }
    (void)hipGetLastError();
    delete e;
    return SP_OK;
}

extern "C" int sp_forward_backward(sp_handle e, const float* x_dev, const float* target_dev, float* y_dev,
                                   float* loss_dev, float* dx_dev, void* const* grad_host_blobs, int B, int S) {
    int rc = check_call(e, B, S);
    if (rc != SP_OK) return rc;
    if (!(e->flags & SP_FLAG_TRAINING)) return fail(e, SP_ERR_STATE, "handle was created without SP_FLAG_TRAINING");
    (void)x_dev; (void)target_dev; (void)y_dev; (void)loss_dev; (void)dx_dev; (void)grad_host_blobs;
    return fail(e, SP_ERR_STATE, "training path not built");
}
