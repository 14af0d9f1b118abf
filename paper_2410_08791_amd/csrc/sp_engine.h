// Engine state behind an sp_handle (internal).
#pragma once
#include <hip/hip_runtime.h>

#include <set>
#include <string>
#include <vector>

#include "sp_host.h"
#include "sp_kernels.h"

struct sp_engine {
    sp_stack_desc desc;
    uint32_t flags = 0;
    sp_plan plan;
    sp::Layout lay;
    sp::Workspace ws;
    sp::Scheduler sched;
    unsigned char* arena = nullptr;   // caller's device arena: [workspace | slot 0 | slot 1 | ...]
    unsigned char* slots = nullptr;
    // A layer streams as `units` units (1 or 3).  Unit u = layer u / units, part u % units: bytes
    // [unit_off[part], + unit_len[part]) of that layer's blob.  Slots 0..n_pinned-1 hold the pinned
    // units at their own sizes, the ring slots follow at plan.slot_bytes each.
    int units = 1, n_units = 0;
    size_t unit_off[3] = {0, 0, 0}, unit_len[3] = {0, 0, 0};
    std::vector<unsigned char*> slot_addr;
    hipStream_t compute = nullptr, h2d = nullptr, d2h = nullptr;
    std::vector<const void*> blobs;   // pinned host weight blobs (never written)
    // Cross-stream fences.  Every copy and every layer compute of a call records
    // its own event (copy_ev[i] / comp_ev[j], i-th copy / j-th compute of the call);
    // layer_loaded / layer_done point at the most recent one for a layer.  With
    // SP_FLAG_TIMING the events carry timestamps and double as the per-layer trace,
    // so tracing adds no operation to either stream.
    // The two pools are rings twice as long as the most operations one call can issue, and a
    // call continues where the previous one stopped: an event that an earlier call recorded --
    // the copy of a layer prefetched for this call, the compute of a slot's last user -- is not
    // recorded again before the call after the next, so a wait on such a handle binds to the
    // operation it was taken for.  A handle is dropped once its one consumer stream has waited
    // on it (that stream is in order, so later operations on it need no second wait); the
    // layers held for good therefore keep no handle into the pool.
    std::vector<hipEvent_t> copy_ev, comp_ev;
    size_t copy_base = 0, comp_base = 0;                 // ring position of the current call's op 0
    hipEvent_t copy_event(int i) const { return copy_ev[(copy_base + (size_t)i) % copy_ev.size()]; }
    hipEvent_t comp_event(int i) const { return comp_ev[(comp_base + (size_t)i) % comp_ev.size()]; }
    int max_copies = 0, max_computes = 0;                // per call
    std::vector<hipEvent_t> layer_loaded, layer_done;
    std::vector<int> layer_loaded_idx, layer_done_idx;   // op index within the current call, -1 = earlier call
    int ci = 0, mi = 0;                                  // ops issued by the current call
    std::vector<int> tr_copy_layer, tr_copy_dep, tr_comp_layer, tr_comp_dep;
    hipEvent_t ev_sync_c = nullptr, ev_sync_h = nullptr;
    // Host run-ahead bound: ring of events, one per enqueued layer op, with the running count
    // of compute-stream packets at each; see throttle() in sp_engine.hip.
    std::vector<hipEvent_t> thr_ev;
    std::vector<uint64_t> thr_at;
    uint64_t thr_head = 0, thr_tail = 0, thr_packets = 0;
    hipEvent_t pass_end_c = nullptr, pass_end_d = nullptr;   // end of the latest training pass on compute / d2h
    bool pass_pending = false;
    int frozen = 0;                             // training: layers below this get no weight gradients
    hipEvent_t grad_ready[sp::kGradSlots] = {}, gslot_free[sp::kGradSlots] = {};
    char gslot_used[sp::kGradSlots] = {};
    int gslot_next = 0;
    std::vector<hipEvent_t> grad_landed;        // per layer: its gradient copy of the latest step (d2h stream)
    std::vector<char> grad_sent;                // per layer: that event has been recorded in the latest step
    hipEvent_t last_grad_copy = nullptr;        // gslot_free event of the most recently submitted gradient copy
    hipEvent_t t0 = nullptr;
    std::vector<hipEvent_t> kt_begin, kt_end;   // ring of event pairs around the largest GEMM
    uint32_t kt_count = 0;                      // pairs recorded since the last sp_get_stats
    uint32_t kt_seen = 0;                       // launches of that GEMM seen (every 4th is timed)
    int kt_m = 0, kt_n = 0, kt_k = 0;
    // counters
    uint64_t calls = 0, stats_h2d_copies = 0, stats_h2d_bytes = 0, stats_d2h_copies = 0, stats_d2h_bytes = 0;
    uint64_t call_h2d_copies = 0, call_h2d_bytes = 0;
    // SP_FLAG_OP_TIMING: event pairs around every kernel launch since the last sp_get_stats
    std::vector<hipEvent_t> op_begin, op_end;
    std::vector<unsigned char> op_tag;
    size_t op_count = 0;
    // debug delays (SP_FLAG_DELAY): upper bound per delay and the running draw counter
    int delay_us = 0;
    uint32_t delay_seq = 0;
    // a call failed after it began to enqueue: residency bookkeeping is ahead of the streams
    bool failed = false;
    std::set<const void*> grad_pinned_ok;       // gradient blobs already verified as pinned host memory
    // training call context
    void* const* grad_blobs = nullptr;
    float* y_out = nullptr;
    std::string error;

    template <class T>
    T* wsp(size_t off) const { return reinterpret_cast<T*>(arena + off); }
};

// One layer forward, residual stream h (fp32 [B*S, d]) updated in place.
// Key/value cache of the layer being run (decode): nullptr fields = plain forward.
struct KvLayer {
    bf16_t* kt = nullptr;   // [B][Hkv][hd][max_len]
    bf16_t* v = nullptr;    // [B][Hkv][max_len][hd]
    int max_len = 0;
    int pos = -1;           // >= 0: one new token per sequence at this position (S == 1)
};
// parts: which of the layer's three blocks to run (bit 0 attention block, bit 1 second norm and
// first FFN projection, bit 2 last FFN projection); w is where the layer blob's byte 0 would be.
int sp_layer_forward(sp_engine* e, const unsigned char* w, float* h, int B, int S, const KvLayer* kv = nullptr,
                     int parts = 7);
// Training forward of layer l: reads its saved input, writes the next layer's.
int sp_layer_forward_train(sp_engine* e, int layer, const unsigned char* w, int B, int S);
// Recompute + backward of layer l; leaves dL/d(input) in the stream-gradient buffer
// and hands the layer's fp32 weight gradients to the device-to-host stream.
int sp_layer_backward(sp_engine* e, int layer, const unsigned char* w, int B, int S);

// Training call phases around the two passes (sp_train.hip).
int sp_train_begin(sp_engine* e, const float* x_dev, int B, int S);
int sp_train_loss(sp_engine* e, const float* target_dev, float* loss_dev, int B, int S);
int sp_train_end(sp_engine* e, float* dx_dev, int B, int S);

int sp_fail(sp_engine* e, int code, const char* fmt, ...);

// A kernel launch of operation kind `tag`, bracketed by timed events when SP_FLAG_OP_TIMING is on
// (until the pool of event pairs is used up; sp_get_stats empties it).
#define SP_OP(e, tag, call)                                                       \
    do {                                                                          \
        const bool _t = (e)->op_count < (e)->op_begin.size();                     \
        if (_t) SP_HIP((e), hipEventRecord((e)->op_begin[(e)->op_count], (e)->compute)); \
        SP_HIP((e), call);                                                        \
        if (_t) {                                                                 \
            SP_HIP((e), hipEventRecord((e)->op_end[(e)->op_count], (e)->compute)); \
            (e)->op_tag[(e)->op_count++] = (unsigned char)(tag);                  \
        }                                                                         \
    } while (0)

#define SP_HIP(e, call)                                                                          \
    do {                                                                                         \
        hipError_t _err = (call);                                                                \
        if (_err != hipSuccess)                                                                  \
            return sp_fail((e), SP_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(_err), \
                           __FILE__, __LINE__);                                                  \
    } while (0)
