// The transfer engine and per-layer executor behind sp_create / sp_forward /
// sp_forward_backward / sp_destroy.
//
// HBM holds n_slots layer-sized slots carved from the caller's arena.  The
// scheduler (sp_host.hip) decides which layer goes to which slot; this file
// turns each decision into stream work:
//   copy(l -> slot):  h2d stream waits for the compute of the slot's previous
//                     user; one hipMemcpyAsync of the whole layer blob; record
//                     a "loaded" event
//   compute(l):       compute stream waits for l's "loaded" event; the layer's
//                     kernels; record a "done" event
// Those two event kinds are the only cross-stream edges (training adds the pair
// that fences the two gradient slots against the device-to-host stream).  An event is always
// recorded (in host order) before anything waits on it.  The host blocks only at
// the run-ahead bound below, at the start of a training step that follows another,
// and in sp_wait_gradient; no device memory is allocated.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <unistd.h>

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

// ---- host run-ahead bound -----------------------------------------------------------
// The host enqueues a whole call in a few milliseconds.  Measured on this runtime: once
// more than roughly 1500 packets (kernels and event records) wait on the compute stream,
// passes take 30-60 % longer in bursts; below that every pass runs at its steady time.  A
// host-side wait is not free either (the copies of the next layers are enqueued late), so
// waits are made rare: when more than kMaxQueuedPackets are unfinished the host sleeps
// until kResumePackets are left, then runs ahead again.
//
// Gradient copies add a second rule, also measured: a device-to-host copy that is
// submitted while an earlier one of the same stream is executing runs at a quarter of
// the link rate (15.8 ms instead of 3.9 ms for 202 MB), and so do all copies submitted
// after it until the host next finds the stream idle; copies submitted while the earlier
// ones are still waiting for their gradients are not affected.  A training step that fits
// the packet bound is therefore enqueued in one go (all its gradient copies are
// submitted before the first one starts), and when a wait inside a backward pass cannot
// be avoided the host also lets the gradient stream drain before it goes on.
// Per-op packet counts are estimates; the ring is longer than any window they allow.
constexpr uint64_t kMaxQueuedPackets = 1400;
constexpr uint64_t kResumePackets = 350;
constexpr size_t kThrottleRing = 256;
constexpr unsigned kPacketsForward = 16, kPacketsForwardTrain = 14, kPacketsBackward = 44;

static int throttle_before(sp_engine* e) {
    auto left_after = [&](uint64_t i) { return e->thr_packets - e->thr_at[i % kThrottleRing]; };
    if (e->thr_tail < e->thr_head &&
        (left_after(e->thr_tail) > kMaxQueuedPackets || e->thr_head - e->thr_tail >= kThrottleRing)) {
        while (e->thr_tail + 1 < e->thr_head && left_after(e->thr_tail + 1) > kResumePackets) e->thr_tail++;
        SP_HIP(e, hipEventSynchronize(e->thr_ev[e->thr_tail % kThrottleRing]));
        e->thr_tail++;
        if (e->last_grad_copy) SP_HIP(e, hipEventSynchronize(e->last_grad_copy));
    }
    return SP_OK;
}

static int throttle_after(sp_engine* e, unsigned packets) {
    e->thr_packets += packets;
    const size_t i = e->thr_head % kThrottleRing;
    SP_HIP(e, hipEventRecord(e->thr_ev[i], e->compute));
    e->thr_at[i] = e->thr_packets;
    e->thr_head++;
    return SP_OK;
}

// ---- debug delays (SP_FLAG_DELAY) -----------------------------------------------------
// Before an operation is enqueued the host sleeps and the operation's stream idles, each for a
// pseudo-random time up to delay_us (a fixed sequence per handle): the two streams and the host
// drift against each other, which a fast run never does.  The idling kernel is bounded and exits.
static int delay_point(sp_engine* e, hipStream_t stream) {
    if (!e->delay_us) return SP_OK;
    uint32_t r = (e->delay_seq++ + 1u) * 2654435761u;
    r ^= r >> 15; r *= 2246822519u; r ^= r >> 13;
    const int host_us = (int)(r % (uint32_t)(e->delay_us + 1));
    const int dev_us = (int)((r >> 11) % (uint32_t)(e->delay_us + 1));
    if (r & 1) SP_HIP(e, spk_launch_spin(stream, dev_us));
    if (r & 2) usleep((useconds_t)host_us);
    return SP_OK;
}

// ---- the sink that enqueues real stream work -------------------------------------
struct HipSink : SchedSink {
    sp_engine* e;
    float* hbuf;        // forward: the residual stream (fp32 [T, d]) being updated in place
    int B, S;
    bool training_fwd = false;
    unsigned char* kv_cache = nullptr;   // decode: the caller's cache, one layer after another
    size_t kv_layer_bytes = 0;
    int kv_max_len = 0, kv_pos = -1;
    explicit HipSink(sp_engine* eng) : e(eng), hbuf(nullptr), B(0), S(0) {}

    int copy(int layer, int slot, int wait_layer) override {
        hipStream_t cs = e->h2d;
        if (e->ci >= e->max_copies) return sp_fail(e, SP_ERR_STATE, "copy event pool exhausted");
        int rc = delay_point(e, cs);
        if (rc != SP_OK) return rc;
        int dep = -1;
        if (e->flags & SP_FLAG_NO_OVERLAP) {
            // Naive comparator: a copy starts only after everything enqueued for compute.
            SP_HIP(e, hipEventRecord(e->ev_sync_c, e->compute));
            SP_HIP(e, hipStreamWaitEvent(cs, e->ev_sync_c, 0));
            dep = e->mi - 1;
        } else if (wait_layer >= 0 && e->layer_done[wait_layer]) {
            SP_HIP(e, hipStreamWaitEvent(cs, e->layer_done[wait_layer], 0));
            dep = e->layer_done_idx[wait_layer];
            e->layer_done[wait_layer] = nullptr;     // the copy stream is in order: one wait serves every later copy
        }
        // `layer` counts units: part q of layer `layer / units`
        const int part = layer % e->units;
        const size_t nbytes = e->unit_len[part];
        unsigned char* dst = e->slot_addr[slot];
        if (e->flags & SP_FLAG_POISON) {
            // bf16 NaN pattern: a read of a slot before its copy lands shows up as NaN output
            SP_HIP(e, spk_launch_fill_u32(cs, reinterpret_cast<uint32_t*>(dst), 0x7FC17FC1u, align_up(nbytes, kSlotAlign) / 4));
        }
        SP_HIP(e, hipMemcpyAsync(dst, static_cast<const unsigned char*>(e->blobs[layer / e->units]) + e->unit_off[part],
                                 nbytes, hipMemcpyHostToDevice, cs));
        hipEvent_t ev = e->copy_event(e->ci);
        SP_HIP(e, hipEventRecord(ev, cs));
        e->layer_loaded[layer] = ev;
        e->layer_loaded_idx[layer] = e->ci;
        e->tr_copy_layer[e->ci] = layer;
        e->tr_copy_dep[e->ci] = dep;
        e->ci++;
        e->stats_h2d_copies++;
        e->stats_h2d_bytes += nbytes;
        e->call_h2d_copies++;
        e->call_h2d_bytes += nbytes;
        return SP_OK;
    }

    int compute(int layer, int slot, int dir, bool /*fresh*/) override {
        hipStream_t st = e->compute;
        if (e->mi >= e->max_computes) return sp_fail(e, SP_ERR_STATE, "compute event pool exhausted");
        int rc = throttle_before(e);
        if (rc != SP_OK) return rc;
        if ((rc = delay_point(e, st)) != SP_OK) return rc;
        int dep = -1;
        if (e->flags & SP_FLAG_NO_OVERLAP) {
            // Naive comparator: compute starts only after every copy enqueued so far.
            SP_HIP(e, hipEventRecord(e->ev_sync_h, e->h2d));
            SP_HIP(e, hipStreamWaitEvent(st, e->ev_sync_h, 0));
            dep = e->ci - 1;
        } else if (e->layer_loaded[layer]) {
            SP_HIP(e, hipStreamWaitEvent(st, e->layer_loaded[layer], 0));
            dep = e->layer_loaded_idx[layer];
            e->layer_loaded[layer] = nullptr;        // the compute stream is in order: later uses need no second wait
        }
        // where byte 0 of the layer blob would lie (a unit slot holds only its part of it: the
        // tensors the part's kernels touch all lie inside the slot)
        const int part = layer % e->units, lyr = layer / e->units;
        const int parts = e->units == 1 ? 7 : 1 << part;
        const unsigned char* w = e->slot_addr[slot] - e->unit_off[part];
        if (dir > 0 && kv_cache) {
            KvLayer kv;
            kv.kt = reinterpret_cast<bf16_t*>(kv_cache + (size_t)lyr * kv_layer_bytes);
            kv.v = reinterpret_cast<bf16_t*>(kv_cache + (size_t)lyr * kv_layer_bytes + kv_layer_bytes / 2);
            kv.max_len = kv_max_len;
            kv.pos = kv_pos;
            rc = sp_layer_forward(e, w, hbuf, B, S, &kv, parts);
        } else if (dir > 0)
            rc = training_fwd ? sp_layer_forward_train(e, layer, w, B, S) : sp_layer_forward(e, w, hbuf, B, S, nullptr, parts);
        else
            rc = sp_layer_backward(e, layer, w, B, S);
        if (rc != SP_OK) return rc;
        hipEvent_t ev = e->comp_event(e->mi);
        SP_HIP(e, hipEventRecord(ev, st));
        e->layer_done[layer] = ev;
        e->layer_done_idx[layer] = e->mi;
        e->tr_comp_layer[e->mi] = layer;
        e->tr_comp_dep[e->mi] = dep;
        e->mi++;
        return throttle_after(e, dir < 0 ? kPacketsBackward : training_fwd ? kPacketsForwardTrain : kPacketsForward);
    }
};

// ---- one decoder / encoder layer, forward, residual stream updated in place -------
int sp_layer_forward(sp_engine* e, const unsigned char* w, float* h, int B, int S, const KvLayer* kv, int parts) {
    const sp_stack_desc& d = e->desc;
    const Layout& L = e->lay;
    hipStream_t st = e->compute;
    const int T = B * S, dm = d.d_model, f = d.d_ffn;
    const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim, nqkv = nq + 2 * nkv;
    auto W = [&](int t) { return reinterpret_cast<const bf16_t*>(w + L.t[t].offset); };
    bf16_t* a = e->wsp<bf16_t>(e->ws.a);
    bf16_t* qkv = e->wsp<bf16_t>(e->ws.qkv);
    bf16_t* o = e->wsp<bf16_t>(e->ws.o);
    bf16_t* z = e->wsp<bf16_t>(e->ws.z);
    const bool dec = d.arch == SP_DECODER_SWIGLU_RMS;
    AttnShape as{B, S, d.n_q_heads, d.n_kv_heads, d.head_dim, d.causal, nqkv};
    GemmArgs g;

    if (parts & 1) {
        // b1: a = norm(h)
        SP_OP(e, SP_OP_NORM, spk_launch_norm(st, h, W(dec ? SP_T_G1 : SP_T_LN1_G), dec ? nullptr : W(SP_T_LN1_B), a, T, dm, d.norm_eps));
        // b2: qkv = a Wqkv^T (+ b)
        g = GemmArgs{a, dm, OP_KMAJOR, W(dec ? SP_T_WQKV : SP_T_E_WQKV), dm, OP_KMAJOR, qkv, nqkv, nullptr, 0,
                     dec ? nullptr : W(SP_T_BQKV), T, nqkv, dm, 0};
        SP_OP(e, SP_OP_GEMM_QKV, spk_launch_gemm(st, EPI_BF16, g));
        // b3: attention.  With a cache the new keys/values are stored first; a decode step then
        // attends its single query per sequence to the cached positions 0..pos.
        if (kv)
            SP_OP(e, SP_OP_ATTENTION, spk_launch_kv_append(st, qkv, nqkv, kv->kt, kv->v, B, S, kv->pos >= 0 ? kv->pos : 0, d.n_q_heads,
                                           d.n_kv_heads, d.head_dim, kv->max_len));
        if (kv && kv->pos >= 0) {
            SP_OP(e, SP_OP_ATTENTION, spk_launch_decode_attention(st, qkv, nqkv, kv->kt, kv->v, o, nq, B, kv->pos + 1, kv->max_len,
                                                  d.n_q_heads, d.n_kv_heads, d.head_dim));
        } else {
            SP_OP(e, SP_OP_ATTENTION, spk_launch_attention(st, qkv, o, nullptr, as));
        }
        // b4: h += o Wo^T (+ b)
        g = GemmArgs{o, nq, OP_KMAJOR, W(dec ? SP_T_WO : SP_T_E_WO), nq, OP_KMAJOR, h, dm, h, dm,
                     dec ? nullptr : W(SP_T_BO), T, dm, nq, 0};
        SP_OP(e, SP_OP_GEMM_O, spk_launch_gemm(st, EPI_RESID_F32, g));
    }
    if (parts & 2) {
        // b5: a = norm(h)
        SP_OP(e, SP_OP_NORM, spk_launch_norm(st, h, W(dec ? SP_T_G2 : SP_T_LN2_G), dec ? nullptr : W(SP_T_LN2_B), a, T, dm, d.norm_eps));
        // every 4th launch of the largest GEMM is bracketed: the two event records cost a gap
        // on the stream, which on a compute-bound stack would show in the step time
        const bool kt = !e->kt_begin.empty() && (e->kt_seen++ % 4 == 0);
        const size_t kti = kt ? e->kt_count % e->kt_begin.size() : 0;
        if (kt) {
            SP_HIP(e, hipEventRecord(e->kt_begin[kti], st));
            e->kt_m = T; e->kt_n = dec ? 2 * f : f; e->kt_k = dm;
        }
        if (dec) {
            // b6+b7: z = silu(a Wg^T) * (a Wu^T), gate applied in the GEMM epilogue
            g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_WGU), dm, OP_KMAJOR, z, f, nullptr, 0, nullptr, T, f, dm, 0};
            SP_OP(e, SP_OP_GEMM_FFN1, spk_launch_gemm(st, EPI_SWIGLU_BF16, g));
            if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
        } else {
            g = GemmArgs{a, dm, OP_KMAJOR, W(SP_T_W1), dm, OP_KMAJOR, z, f, nullptr, 0, W(SP_T_B1), T, f, dm, 0};
            SP_OP(e, SP_OP_GEMM_FFN1, spk_launch_gemm(st, EPI_GELU_BF16, g));
            if (kt) { SP_HIP(e, hipEventRecord(e->kt_end[kti], st)); e->kt_count++; }
        }
    }
    if (parts & 4) {
        if (dec) {
            // b8: h += z Wd^T
            g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_WD), f, OP_KMAJOR, h, dm, h, dm, nullptr, T, dm, f, 0};
            SP_OP(e, SP_OP_GEMM_FFN2, spk_launch_gemm(st, EPI_RESID_F32, g));
        } else {
            g = GemmArgs{z, f, OP_KMAJOR, W(SP_T_W2), f, OP_KMAJOR, h, dm, h, dm, W(SP_T_B2), T, dm, f, 0};
            SP_OP(e, SP_OP_GEMM_FFN2, spk_launch_gemm(st, EPI_RESID_F32, g));
        }
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
    const int mode = training ? ((cfg->flags & SP_FLAG_KEEP_ACTIVATIONS) ? 2 : 1) : 0;
    if (!training && (cfg->flags & SP_FLAG_KEEP_ACTIVATIONS))
        return fail(nullptr, SP_ERR_INVALID_ARG, "SP_FLAG_KEEP_ACTIVATIONS needs SP_FLAG_TRAINING");
    if (cfg->h2d_stream == cfg->compute_stream) return fail(nullptr, SP_ERR_INVALID_ARG, "h2d_stream must differ from compute_stream");
    if (training && (!cfg->d2h_stream || cfg->d2h_stream == cfg->compute_stream || cfg->d2h_stream == cfg->h2d_stream))
        return fail(nullptr, SP_ERR_INVALID_ARG, "training needs a d2h_stream distinct from the other two");
    if (desc->n_layers > 4096) return fail(nullptr, SP_ERR_INVALID_ARG, "n_layers > 4096");
    if (cfg->frozen_layers < 0 || cfg->frozen_layers > desc->n_layers || (cfg->frozen_layers && !training))
        return fail(nullptr, SP_ERR_INVALID_ARG, "frozen_layers must be in 0..n_layers and needs SP_FLAG_TRAINING");
    const int units = cfg->units_per_layer ? cfg->units_per_layer : 1;
    if (units != 1 && units != 3) return fail(nullptr, SP_ERR_INVALID_ARG, "units_per_layer must be 0, 1 or 3");
    if (units != 1 && training) return fail(nullptr, SP_ERR_INVALID_ARG, "units_per_layer = 3 is for forward-only handles");
    if ((cfg->flags & SP_FLAG_DELAY) && (cfg->delay_us < 0 || cfg->delay_us > SPK_SPIN_MAX_US))
        return fail(nullptr, SP_ERR_INVALID_ARG, "delay_us must be in 0..%d", SPK_SPIN_MAX_US);
    sp_plan plan;
    int rc = make_plan(desc, units, cfg->resident_window_k, cfg->prefetch_depth_p, cfg->pinned_layers,
                       cfg->gpu_budget_bytes, mode, &plan);
    if (rc == SP_ERR_BUDGET) {
        return fail(nullptr, rc, "gpu_budget_bytes=%llu cannot hold the workspace (%llu) plus one slot (%llu)",
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
    e->frozen = training ? cfg->frozen_layers : 0;
    e->plan = plan;
    make_layout(desc, &e->lay);
    make_workspace(desc, e->lay, mode, &e->ws);
    e->arena = static_cast<unsigned char*>(cfg->device_arena);
    e->slots = e->arena + e->ws.total;
    e->units = units;
    e->n_units = desc->n_layers * units;
    for (int q = 0; q < units; ++q) unit_range(desc, e->lay, units, q, &e->unit_off[q], &e->unit_len[q]);
    {
        // pinned units first, each at its own size, then the ring of equal slots
        unsigned char* at = e->slots;
        e->slot_addr.resize(plan.n_slots);
        for (int s = 0; s < plan.n_slots; ++s) {
            e->slot_addr[s] = at;
            at += s < plan.n_pinned ? align_up(e->unit_len[s % units], kSlotAlign) : plan.slot_bytes;
        }
    }
    e->compute = static_cast<hipStream_t>(cfg->compute_stream);
    e->h2d = static_cast<hipStream_t>(cfg->h2d_stream);
    e->d2h = static_cast<hipStream_t>(cfg->d2h_stream);
    e->blobs.assign(blobs, blobs + desc->n_layers);
    const int L = e->n_units;      // what the scheduler calls a layer: a unit
    const bool timing = cfg->flags & SP_FLAG_TIMING;
    // a call issues at most 2L + n_slots copies and 2L computes (forward + backward); the event
    // rings hold two calls' worth
    e->max_copies = (training ? 2 : 1) * L + plan.n_slots + 1;
    e->max_computes = (training ? 2 : 1) * L + 1;
    e->copy_ev.assign(2 * (size_t)e->max_copies, nullptr);
    e->comp_ev.assign(2 * (size_t)e->max_computes, nullptr);
    e->tr_copy_layer.assign(e->max_copies, -1);
    e->tr_copy_dep.assign(e->max_copies, -1);
    e->tr_comp_layer.assign(e->max_computes, -1);
    e->tr_comp_dep.assign(e->max_computes, -1);
    e->layer_loaded.assign(L, nullptr);
    e->layer_done.assign(L, nullptr);
    e->layer_loaded_idx.assign(L, -1);
    e->layer_done_idx.assign(L, -1);
    const unsigned evflags = timing ? hipEventDefault : hipEventDisableTiming;
    auto mk = [&](hipEvent_t* ev, unsigned fl) { return hipEventCreateWithFlags(ev, fl); };
    hipError_t he = hipSuccess;
    for (size_t i = 0; i < e->copy_ev.size() && he == hipSuccess; ++i) he = mk(&e->copy_ev[i], evflags);
    for (size_t i = 0; i < e->comp_ev.size() && he == hipSuccess; ++i) he = mk(&e->comp_ev[i], evflags);
    if (he == hipSuccess) he = mk(&e->ev_sync_c, hipEventDisableTiming);
    if (he == hipSuccess) he = mk(&e->ev_sync_h, hipEventDisableTiming);
    e->thr_ev.assign(kThrottleRing, nullptr);
    e->thr_at.assign(kThrottleRing, 0);
    for (size_t i = 0; i < kThrottleRing && he == hipSuccess; ++i) he = mk(&e->thr_ev[i], hipEventDisableTiming);
    if (he == hipSuccess && training) he = mk(&e->pass_end_c, hipEventDisableTiming);
    if (he == hipSuccess && training) he = mk(&e->pass_end_d, hipEventDisableTiming);
    for (int i = 0; i < kGradSlots && he == hipSuccess; ++i) {
        he = mk(&e->grad_ready[i], hipEventDisableTiming);
        if (he == hipSuccess) he = mk(&e->gslot_free[i], hipEventDisableTiming);
    }
    if (training) {
        e->grad_landed.assign(L, nullptr);
        e->grad_sent.assign(L, 0);
        for (int i = 0; i < L && he == hipSuccess; ++i) he = mk(&e->grad_landed[i], hipEventDisableTiming);
    }
    if (he == hipSuccess && timing) he = mk(&e->t0, hipEventDefault);
    if (he == hipSuccess && (cfg->flags & (SP_FLAG_TIMING | SP_FLAG_KERNEL_TIMING))) {
        e->kt_begin.assign(2048, nullptr);
        e->kt_end.assign(2048, nullptr);
        for (size_t i = 0; i < e->kt_begin.size() && he == hipSuccess; ++i) {
            he = mk(&e->kt_begin[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->kt_end[i], hipEventDefault);
        }
    }
    if (he == hipSuccess && (cfg->flags & SP_FLAG_OP_TIMING)) {
        // a training step of the deepest stacks in use launches about 3000 kernels
        e->op_begin.assign(8192, nullptr);
        e->op_end.assign(8192, nullptr);
        e->op_tag.assign(8192, 0);
        for (size_t i = 0; i < e->op_begin.size() && he == hipSuccess; ++i) {
            he = mk(&e->op_begin[i], hipEventDefault);
            if (he == hipSuccess) he = mk(&e->op_end[i], hipEventDefault);
        }
    }
    if (he != hipSuccess) {
        fail(nullptr, SP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(he));
        destroy_engine(e);
        return SP_ERR_HIP;
    }
    const bool naive = cfg->flags & SP_FLAG_NO_OVERLAP;
    e->sched.reset(L, plan.n_slots, naive ? plan.n_slots - plan.n_pinned : plan.p_eff, plan.n_pinned);
    if (cfg->flags & SP_FLAG_DELAY) e->delay_us = cfg->delay_us ? cfg->delay_us : 200;
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

// A pass that fails after it began leaves the scheduler's residency ahead of what the streams
// hold (a layer recorded as resident whose copy was never issued): the handle refuses further
// passes.  The first error's text stays in front for sp_last_error.
static int mark_failed(sp_engine* e, int rc) {
    if (rc != SP_OK && !e->failed) {
        e->failed = true;
        e->error = "handle FAILED mid-pass (only sp_destroy is left): " + e->error;
    }
    return rc;
}

static int check_call(sp_engine* e, int B, int S) {
    if (!e) return SP_ERR_INVALID_ARG;
    if (!is_live(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (destroyed or never created)");
    if (e->failed) return SP_ERR_STATE;          // e->error keeps the first failure's text
    if (B < 1 || S < 1 || B > e->desc.max_batch || S > e->desc.max_seq)
        return fail(e, SP_ERR_SHAPE, "B=%d S=%d outside 1..%d x 1..%d", B, S, e->desc.max_batch, e->desc.max_seq);
    return SP_OK;
}

static int begin_call(sp_engine* e) {
    e->call_h2d_copies = e->call_h2d_bytes = 0;
    e->copy_base = (e->copy_base + (size_t)e->ci) % e->copy_ev.size();
    e->comp_base = (e->comp_base + (size_t)e->mi) % e->comp_ev.size();
    e->ci = e->mi = 0;
    std::fill(e->layer_loaded_idx.begin(), e->layer_loaded_idx.end(), -1);
    std::fill(e->layer_done_idx.begin(), e->layer_done_idx.end(), -1);
    if (e->flags & SP_FLAG_TIMING) SP_HIP(e, hipEventRecord(e->t0, e->compute));
    return SP_OK;
}

// bytes of one layer's cache: keys and values, bf16
static size_t kv_layer_bytes(const sp_stack_desc& d, int batch, int max_len) {
    return (size_t)2 * batch * d.n_kv_heads * d.head_dim * max_len * sizeof(bf16_t);
}

// One forward pass, arguments already checked: from here on a failure leaves the handle FAILED.
static int enqueue_forward(sp_engine* e, const float* x_dev, float* y_dev, int B, int S, void* kv_cache_dev,
                           int max_len, int pos) {
    int rc;
    if ((rc = begin_call(e)) != SP_OK) return rc;
    SP_OP(e, SP_OP_COPY, spk_launch_copy_f32(e->compute, x_dev, y_dev, (size_t)B * S * e->desc.d_model));
    HipSink sink(e);
    sink.hbuf = y_dev;
    sink.B = B;
    sink.S = S;
    if (kv_cache_dev) {
        sink.kv_cache = static_cast<unsigned char*>(kv_cache_dev);
        sink.kv_layer_bytes = kv_layer_bytes(e->desc, B, max_len);
        sink.kv_max_len = max_len;
        sink.kv_pos = pos;
    }
    const bool wrap = (e->flags & SP_FLAG_WRAP_PREFETCH) && !(e->flags & SP_FLAG_TRAINING);
    if ((rc = e->sched.run_pass(+1, wrap, sink)) != SP_OK) {
        if (e->error.empty()) sp_fail(e, rc, "scheduler refused the pass");
        return rc;
    }
    e->calls++;
    return SP_OK;
}

extern "C" int sp_forward(sp_handle e, const float* x_dev, float* y_dev, int B, int S) {
    int rc = check_call(e, B, S);
    if (rc != SP_OK) return rc;
    if (!x_dev || !y_dev) return fail(e, SP_ERR_INVALID_ARG, "x_dev / y_dev is NULL");
    if (((uintptr_t)x_dev | (uintptr_t)y_dev) & 15) return fail(e, SP_ERR_INVALID_ARG, "x_dev / y_dev must be 16-byte aligned");
    return mark_failed(e, enqueue_forward(e, x_dev, y_dev, B, S, nullptr, 0, -1));
}

extern "C" size_t sp_kv_cache_bytes(const sp_stack_desc* desc, int batch, int max_len) {
    const char* why = nullptr;
    if (!desc || validate_desc(desc, &why) != SP_OK || batch < 1 || max_len < 2 || (max_len & 7) ||
        max_len > kDecodeMaxLen)
        return 0;
    return (size_t)desc->n_layers * kv_layer_bytes(*desc, batch, max_len);
}

static int cached_forward(sp_engine* e, const float* x_dev, float* y_dev, void* kv_cache_dev, int B, int S, int pos,
                          int max_len) {
    const sp_stack_desc& d = e->desc;
    if (d.arch != SP_DECODER_SWIGLU_RMS || !d.causal || (d.head_dim != 64 && d.head_dim != 128))
        return fail(e, SP_ERR_STATE, "the key/value cache needs a causal decoder stack with head_dim 64 or 128");
    if (e->flags & SP_FLAG_TRAINING) return fail(e, SP_ERR_STATE, "handle was created for training");
    if (!x_dev || !y_dev || !kv_cache_dev) return fail(e, SP_ERR_INVALID_ARG, "NULL argument");
    if (((uintptr_t)x_dev | (uintptr_t)y_dev | (uintptr_t)kv_cache_dev) & 15)
        return fail(e, SP_ERR_INVALID_ARG, "x_dev / y_dev / kv_cache_dev must be 16-byte aligned");
    if (max_len < 2 || (max_len & 7) || max_len > kDecodeMaxLen)
        return fail(e, SP_ERR_SHAPE, "max_len=%d must be a multiple of 8 in 8..%d", max_len, kDecodeMaxLen);
    const int first = pos >= 0 ? pos : 0;
    if (first + S > max_len) return fail(e, SP_ERR_SHAPE, "positions %d..%d exceed max_len=%d", first, first + S - 1, max_len);
    return mark_failed(e, enqueue_forward(e, x_dev, y_dev, B, S, kv_cache_dev, max_len, pos));
}

extern "C" int sp_prefill(sp_handle e, const float* x_dev, float* y_dev, void* kv_cache_dev, int B, int S,
                          int max_len) {
    int rc = check_call(e, B, S);
    if (rc != SP_OK) return rc;
    return cached_forward(e, x_dev, y_dev, kv_cache_dev, B, S, -1, max_len);
}

extern "C" int sp_decode(sp_handle e, const float* x_dev, float* y_dev, void* kv_cache_dev, int B, int pos,
                         int max_len) {
    int rc = check_call(e, B, 1);
    if (rc != SP_OK) return rc;
    if (pos < 0) return fail(e, SP_ERR_SHAPE, "pos=%d is negative", pos);
    return cached_forward(e, x_dev, y_dev, kv_cache_dev, B, 1, pos, max_len);
}

static int enqueue_training_step(sp_engine* e, const float* x_dev, const float* target_dev, float* y_dev,
                                 float* loss_dev, float* dx_dev, void* const* grad_host_blobs, int B, int S);

extern "C" int sp_forward_backward(sp_handle e, const float* x_dev, const float* target_dev, float* y_dev,
                                   float* loss_dev, float* dx_dev, void* const* grad_host_blobs, int B, int S) {
    int rc = check_call(e, B, S);
    if (rc != SP_OK) return rc;
    if (!(e->flags & SP_FLAG_TRAINING)) return fail(e, SP_ERR_STATE, "handle was created without SP_FLAG_TRAINING");
    if (!x_dev || !target_dev || !loss_dev || !grad_host_blobs) return fail(e, SP_ERR_INVALID_ARG, "NULL argument");
    if (((uintptr_t)x_dev | (uintptr_t)target_dev | (uintptr_t)y_dev | (uintptr_t)dx_dev) & 15)
        return fail(e, SP_ERR_INVALID_ARG, "device tensors must be 16-byte aligned");
    for (int l = e->frozen; l < e->desc.n_layers; ++l) {
        const void* gb = grad_host_blobs[l];
        if (!gb) return fail(e, SP_ERR_INVALID_ARG, "grad_host_blobs[%d] is NULL", l);
        if (e->grad_pinned_ok.count(gb)) continue;       // verified by an earlier step
        hipPointerAttribute_t at;
        hipError_t pe = hipPointerGetAttributes(&at, gb);
        if (pe != hipSuccess || at.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            return fail(e, SP_ERR_NOT_PINNED, "grad_host_blobs[%d] is not pinned host memory", l);
        }
        e->grad_pinned_ok.insert(gb);
    }
    return mark_failed(e, enqueue_training_step(e, x_dev, target_dev, y_dev, loss_dev, dx_dev, grad_host_blobs, B, S));
}

static int enqueue_training_step(sp_engine* e, const float* x_dev, const float* target_dev, float* y_dev,
                                 float* loss_dev, float* dx_dev, void* const* grad_host_blobs, int B, int S) {
    int rc;
    // One training pass in flight: the host waits here until the previous pass has
    // delivered its last gradient.  Its consumer (the host-side optimizer) needs that
    // point anyway, and copies enqueued more than a pass ahead were measured to drop
    // the device-to-host engine to a fraction of the link rate.
    if (e->pass_pending) {
        SP_HIP(e, hipEventSynchronize(e->pass_end_d));
        SP_HIP(e, hipEventSynchronize(e->pass_end_c));
        e->pass_pending = false;
    }
    if ((rc = begin_call(e)) != SP_OK) return rc;
    std::fill(e->grad_sent.begin(), e->grad_sent.end(), 0);
    e->grad_blobs = grad_host_blobs;
    e->y_out = y_dev;
    if ((rc = sp_train_begin(e, x_dev, B, S)) != SP_OK) return rc;
    HipSink sink(e);
    sink.B = B;
    sink.S = S;
    sink.training_fwd = true;
    if ((rc = e->sched.run_pass(+1, false, sink)) != SP_OK) return rc;
    if ((rc = sp_train_loss(e, target_dev, loss_dev, B, S)) != SP_OK) return rc;
    sink.training_fwd = false;
    // without dx nothing below the frozen layers needs a gradient: the backward stops above them
    if ((rc = e->sched.run_pass(-1, false, sink, dx_dev ? 0 : e->frozen)) != SP_OK) return rc;
    if ((rc = sp_train_end(e, dx_dev, B, S)) != SP_OK) return rc;
    SP_HIP(e, hipEventRecord(e->pass_end_c, e->compute));
    SP_HIP(e, hipEventRecord(e->pass_end_d, e->d2h));
    e->pass_pending = true;
    e->calls++;
    return SP_OK;
}

extern "C" int sp_wait_gradient(sp_handle e, int layer) {
    if (!e) return SP_ERR_INVALID_ARG;
    if (!is_live(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (destroyed or never created)");
    if (e->failed) return SP_ERR_STATE;
    if (!(e->flags & SP_FLAG_TRAINING)) return fail(e, SP_ERR_STATE, "handle was created without SP_FLAG_TRAINING");
    if (layer < 0 || layer >= e->desc.n_layers) return fail(e, SP_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!e->grad_sent[layer])
        return fail(e, SP_ERR_STATE, "layer %d has no gradient on its way (frozen, or no training step since create)", layer);
    SP_HIP(e, hipEventSynchronize(e->grad_landed[layer]));
    return SP_OK;
}

extern "C" int sp_weights_updated(sp_handle e, int layer) {
    if (!e) return SP_ERR_INVALID_ARG;
    if (!is_live(e)) return fail(nullptr, SP_ERR_STATE, "handle is not live (destroyed or never created)");
    if (e->failed) return SP_ERR_STATE;
    const int L = e->desc.n_layers;
    if (layer < -1 || layer >= L) return fail(e, SP_ERR_INVALID_ARG, "layer %d out of range", layer);
    const int lo = layer < 0 ? 0 : layer, hi = layer < 0 ? L : layer + 1;
    for (int u = lo * e->units; u < hi * e->units; ++u) e->sched.invalidate(u);
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
    if (!(e->flags & (SP_FLAG_TIMING | SP_FLAG_KERNEL_TIMING | SP_FLAG_OP_TIMING)) || e->calls == 0) return SP_OK;
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
    for (size_t i = 0; i < e->op_count; ++i) {
        float ms = 0;
        SP_HIP(e, hipEventElapsedTime(&ms, e->op_begin[i], e->op_end[i]));
        out->op_ms[e->op_tag[i]] += ms;
        out->op_launches[e->op_tag[i]]++;
    }
    e->op_count = 0;
    if (!(e->flags & SP_FLAG_TIMING)) return SP_OK;
    // Per-op trace of the most recent call from the fence events' timestamps.  An op
    // begins when its stream's previous op has ended and its dependency is met.
    const int nc = e->ci, nm = e->mi;
    std::vector<float> tc(nc), tm(nm), cb(nc), mb(nm);
    for (int i = 0; i < nc; ++i) SP_HIP(e, hipEventElapsedTime(&tc[i], e->t0, e->copy_event(i)));
    for (int j = 0; j < nm; ++j) SP_HIP(e, hipEventElapsedTime(&tm[j], e->t0, e->comp_event(j)));
    for (int i = 0; i < nc; ++i) {
        float b = i > 0 ? tc[i - 1] : std::min(0.f, tc[i]);
        const int dep = e->tr_copy_dep[i];
        if (dep >= 0 && dep < nm) b = std::max(b, tm[dep]);
        cb[i] = std::min(b, tc[i]);
    }
    for (int j = 0; j < nm; ++j) {
        float b = j > 0 ? tm[j - 1] : 0.f;
        const int dep = e->tr_comp_dep[j];
        if (dep >= 0 && dep < nc) b = std::max(b, tc[dep]);
        mb[j] = std::min(b, tm[j]);
    }
    std::vector<std::pair<float, float>> comp(nm);
    float tmin = 1e30f, tmax = -1e30f;
    const int n = std::min(nm, (int)SP_MAX_TRACE_LAYERS);
    out->n_timed = n;
    out->n_ops = nm;
    for (int j = 0; j < nm; ++j) {
        comp[j] = {mb[j], tm[j]};
        out->compute_busy_ms += tm[j] - mb[j];
        tmin = std::min(tmin, mb[j]);
        tmax = std::max(tmax, tm[j]);
        if (j < n) {
            out->comp_begin_ms[j] = mb[j];
            out->comp_end_ms[j] = tm[j];
            out->copy_begin_ms[j] = out->copy_end_ms[j] = -1.f;
            const int dep = e->tr_comp_dep[j];
            if (dep >= 0 && dep < nc && e->tr_copy_layer[dep] == e->tr_comp_layer[j]) {
                out->copy_begin_ms[j] = cb[dep];
                out->copy_end_ms[j] = tc[dep];
            }
        }
    }
    for (int i = 0; i < nc; ++i) {
        out->copy_busy_ms += tc[i] - cb[i];
        for (auto& iv : comp) {
            const float lo = std::max(cb[i], iv.first), hi = std::min(tc[i], iv.second);
            if (hi > lo) out->copy_hidden_ms += hi - lo;
        }
        tmin = std::min(tmin, cb[i]);
        tmax = std::max(tmax, tc[i]);
    }
    out->wall_ms = (nm || nc) ? tmax - tmin : 0.f;
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
    for (auto ev : e->copy_ev) kill(ev);
    for (auto ev : e->comp_ev) kill(ev);
    for (auto ev : e->kt_begin) kill(ev);
    for (auto ev : e->kt_end) kill(ev);
    for (auto ev : e->op_begin) kill(ev);
    for (auto ev : e->op_end) kill(ev);
    kill(e->ev_sync_c);
    kill(e->ev_sync_h);
    for (auto ev : e->thr_ev) kill(ev);
    kill(e->pass_end_c);
    kill(e->pass_end_d);
    kill(e->t0);
    for (int i = 0; i < kGradSlots; ++i) { kill(e->grad_ready[i]); kill(e->gslot_free[i]); }
    for (auto ev : e->grad_landed) kill(ev);
    (void)hipGetLastError();
    delete e;
    return SP_OK;
}
