// Layout, workspace, slot-count policy, window scheduler and the host-only
// C entry points (no device needed for anything in this file).
#include "sp_host.h"
#include "sp_limits.h"

#include <string.h>

#include <algorithm>

namespace sp {

constexpr int kNormBwdBlocks = SPK_NORM_BWD_BLOCKS;
static_assert(SPK_MSE_PARTS <= 1024, "loss partials share the tail of the partial-sum buffer");

int validate_desc(const sp_stack_desc* d, const char** why) {
    const char* w = nullptr;
    if (!d) w = "desc is NULL";
    else if (d->struct_size != sizeof(sp_stack_desc)) w = "desc.struct_size mismatch";
    else if (d->arch != SP_DECODER_SWIGLU_RMS && d->arch != SP_ENCODER_GELU_LN) w = "unknown arch";
    else if (d->n_layers < 1) w = "n_layers < 1";
    else if (d->d_model < 64 || d->d_model % 64 || d->d_model > 8192) w = "d_model must be a multiple of 64 in [64, 8192]";
    else if (d->head_dim != 64 && d->head_dim != 80 && d->head_dim != 128) w = "head_dim must be 64, 80 or 128";
    else if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) w = "n_kv_heads must divide n_q_heads";
    else if ((d->n_q_heads * d->head_dim) % 64) w = "n_q_heads*head_dim must be a multiple of 64";
    // the fused q/k/v width is a contraction length of the backward pass (da = dqkv Wqkv)
    else if (((d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim) % 64) w = "(n_q_heads + 2 n_kv_heads)*head_dim must be a multiple of 64";
    else if (d->d_ffn < 64 || d->d_ffn % 64) w = "d_ffn must be a multiple of 64";
    else if (d->max_batch < 1 || d->max_seq < 1) w = "max_batch/max_seq < 1";
    else if ((int64_t)d->max_batch * d->max_seq > (1 << 24)) w = "max_batch*max_seq too large";
    else if (!(d->norm_eps > 0.f)) w = "norm_eps must be positive";
    else if (d->arch == SP_ENCODER_GELU_LN && d->causal) w = "encoder layers are bidirectional";
    if (why) *why = w;
    return w ? SP_ERR_INVALID_ARG : SP_OK;
}

int make_layout(const sp_stack_desc* d, Layout* out) {
    int rc = validate_desc(d, nullptr);
    if (rc != SP_OK) return rc;
    const int dm = d->d_model, f = d->d_ffn;
    const int nq = d->n_q_heads * d->head_dim, nkv = d->n_kv_heads * d->head_dim;
    const int nqkv = nq + 2 * nkv;
    struct RC { int r, c; };
    RC shapes[kMaxTensors];
    int n;
    if (d->arch == SP_DECODER_SWIGLU_RMS) {
        const RC s[] = {{1, dm}, {nqkv, dm}, {dm, nq}, {1, dm}, {2 * f, dm}, {dm, f}};
        n = SP_DECODER_TENSORS;
        memcpy(shapes, s, sizeof(s));
    } else {
        const RC s[] = {{1, dm}, {1, dm}, {nqkv, dm}, {1, nqkv}, {dm, nq}, {1, dm},
                        {1, dm}, {1, dm}, {f, dm},    {1, f},    {dm, f},  {1, dm}};
        n = SP_ENCODER_TENSORS;
        memcpy(shapes, s, sizeof(s));
    }
    size_t off = 0;
    out->n_tensors = n;
    for (int i = 0; i < n; ++i) {
        out->t[i].offset = off;
        out->t[i].rows = shapes[i].r;
        out->t[i].cols = shapes[i].c;
        out->t[i].elems = (size_t)shapes[i].r * shapes[i].c;
        off = align_up(off + out->t[i].elems * 2, kTensorAlign);
    }
    out->blob_bytes = off;
    out->grad_bytes = off * 2;
    return SP_OK;
}

void make_workspace(const sp_stack_desc* d, const Layout& lay, int training, Workspace* ws) {
    memset(ws, 0, sizeof(*ws));
    const size_t T = (size_t)d->max_batch * d->max_seq;
    const size_t Tp = training ? align_up(T, 64) : T;
    ws->t_pad = (int)Tp;
    const size_t dm = d->d_model, f = d->d_ffn;
    const size_t nq = (size_t)d->n_q_heads * d->head_dim, nkv = (size_t)d->n_kv_heads * d->head_dim;
    const size_t nqkv = nq + 2 * nkv;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, kTensorAlign); return o; };
    // per-layer activation set (one shared set, or one per layer when activations are kept)
    ws->a = take(Tp * dm * 2);
    ws->qkv = take(Tp * nqkv * 2);
    ws->o = take(Tp * nq * 2);
    // [gate | up] resp. the MLP pre-activation: only the backward needs them in memory (the
    // forward applies SwiGLU / GELU in the producing GEMM's epilogue and stores z alone)
    ws->gu = training ? take(Tp * (d->arch == SP_DECODER_SWIGLU_RMS ? 2 * f : f) * 2) : off;
    ws->z = take(Tp * f * 2);
    if (training) {
        ws->m = take(Tp * dm * 2);
        ws->h1 = take(T * dm * 4);
        ws->lse = take((size_t)d->max_batch * d->n_q_heads * d->max_seq * 4);
    }
    ws->set_stride = 0;
    if (training == 2) {
        ws->set_stride = off;                       // sets of layers 1..L-1 follow set 0
        off += ws->set_stride * (size_t)(d->n_layers - 1);
    }
    if (training) {
        ws->xs = take((size_t)d->n_layers * T * dm * 4);
        ws->delta = take((size_t)d->max_batch * d->n_q_heads * d->max_seq * 4);
        ws->dh = take(T * dm * 4);
        ws->da = take(T * dm * 4);
        ws->dhb = take(Tp * dm * 2);
        ws->dqkv = take(Tp * nqkv * 2);
        ws->dob = take(Tp * nq * 2);
        ws->dz = take(Tp * f * 2);
        // partial rows of the two-stage column reductions: gain gradients (d columns), and
        // for the encoder gain + bias (2d) and the linear maps' bias gradients (up to nqkv or f)
        const size_t pcols = d->arch == SP_DECODER_SWIGLU_RMS ? dm : std::max(std::max(2 * dm, nqkv), f);
        ws->part = take(((size_t)kNormBwdBlocks * pcols + 1024) * 4);
        off = align_up(off, kSlotAlign);
        for (int i = 0; i < kGradSlots; ++i) ws->gslot[i] = take(align_up(lay.grad_bytes, kSlotAlign));
    }
    ws->total = align_up(off, kSlotAlign);
}

int unit_range(const sp_stack_desc* d, const Layout& lay, int units, int part, size_t* off, size_t* len) {
    if (units == 1 && part == 0) { *off = 0; *len = lay.blob_bytes; return SP_OK; }
    if (units != 3 || part < 0 || part > 2) return SP_ERR_INVALID_ARG;
    // blob order: [attention block | second norm + first FFN projection | last FFN projection]
    const bool dec = d->arch == SP_DECODER_SWIGLU_RMS;
    const size_t cut1 = lay.t[dec ? SP_T_G2 : SP_T_LN2_G].offset, cut2 = lay.t[dec ? SP_T_WD : SP_T_W2].offset;
    const size_t b[4] = {0, cut1, cut2, lay.blob_bytes};
    *off = b[part];
    *len = b[part + 1] - b[part];
    return SP_OK;
}

int make_plan(const sp_stack_desc* d, int units, int k, int p, int pinned, uint64_t budget, int training, sp_plan* out) {
    if (!out) return SP_ERR_INVALID_ARG;
    memset(out, 0, sizeof(*out));
    Layout lay;
    int rc = make_layout(d, &lay);
    if (rc != SP_OK) return rc;
    if (units == 0) units = 1;
    if ((units != 1 && units != 3) || (units != 1 && training)) return SP_ERR_INVALID_ARG;
    if (k < 1 || p < 1 || pinned < SP_PIN_AUTO) return SP_ERR_INVALID_ARG;
    Workspace ws;
    make_workspace(d, lay, training, &ws);
    size_t ubytes[3] = {0, 0, 0};      // each part's size in the arena
    for (int q = 0; q < units; ++q) {
        size_t off, len;
        unit_range(d, lay, units, q, &off, &len);
        ubytes[q] = align_up(len, kSlotAlign);
        out->slot_bytes = std::max<uint64_t>(out->slot_bytes, ubytes[q]);
    }
    out->units_per_layer = units;
    out->workspace_bytes = ws.total;
    if (budget < ws.total + out->slot_bytes) return SP_ERR_BUDGET;
    const int64_t L = (int64_t)d->n_layers * units;      // units in the stack
    const uint64_t room = budget - ws.total;
    const int64_t cap = std::min<int64_t>(L, (int64_t)std::min<uint64_t>(room / out->slot_bytes, 1u << 30));
    // the streaming window comes first; pinned units take what the budget leaves
    const int64_t window = std::min<int64_t>((int64_t)k + p, cap);
    uint64_t left = room - (uint64_t)window * out->slot_bytes, pinned_bytes = 0;
    int64_t r = 0;
    while (r < L && (pinned == SP_PIN_AUTO || r < pinned) && ubytes[r % units] <= left) {
        left -= ubytes[r % units];
        pinned_bytes += ubytes[r % units];
        ++r;
    }
    int64_t n = window + r;
    if (n >= L) {
        if ((uint64_t)L * out->slot_bytes <= room) {
            n = L; r = 0; pinned_bytes = 0;        // everything fits uniform slots: nothing streams, nothing to pin
        } else {
            // fits only with the pinned units at their own sizes: keep one unit streaming
            while (r > 0 && window + r >= L) { --r; pinned_bytes -= ubytes[r % units]; }
            n = window + r;
        }
    }
    out->n_slots = (int)n;
    out->n_pinned = (int)r;
    out->pinned_bytes = pinned_bytes;
    const int64_t ring = n - r;
    out->p_eff = (int)std::min<int64_t>(p, std::max<int64_t>(ring - 1, 1));
    out->k_eff = (int)std::max<int64_t>(ring - out->p_eff, 1);
    out->fully_resident = n == L;
    out->arena_bytes_used = ws.total + pinned_bytes + (uint64_t)ring * out->slot_bytes;
    return SP_OK;
}

// ---- scheduler ---------------------------------------------------------------
void Scheduler::reset(int n_layers, int n_slots, int group, int n_pinned) {
    n_layers_ = n_layers;
    n_slots_ = n_slots;
    group_ = std::max(1, group);
    // pinned layers only make sense next to a streaming ring of at least one slot
    n_pinned_ = (n_slots >= n_layers) ? 0 : std::max(0, std::min(n_pinned, n_slots - 1));
    slot_layer_.assign(n_slots, -1);
    slot_last_.assign(n_slots, -1);
    layer_slot_.assign(n_layers, -1);
    fresh_.assign(n_layers, 0);
}

void Scheduler::invalidate(int layer) {
    if (layer < 0 || layer >= n_layers_) return;
    const int s = layer_slot_[layer];
    if (s >= 0) {
        slot_layer_[s] = -1;
        layer_slot_[layer] = -1;
    }
    fresh_[layer] = 0;
}

int Scheduler::run_pass(int dir, bool wrap, SchedSink& sink, int lo) {
    const int L = n_layers_, N = n_slots_, R = n_pinned_;
    if (lo < 0 || lo > L) return SP_ERR_INVALID_ARG;
    int rc;
    // Layers 0..R-1 are pinned: slot l holds layer l from its first use on and is never
    // refilled.  The other layers stream through the ring of slots R..N-1.
    std::vector<int> order;            // streamed layers in the order this pass needs them
    order.reserve(L - R);
    for (int i = 0; i < L; ++i) {
        const int l = dir > 0 ? i : L - 1 - i;
        if (l >= R && l >= lo) order.push_back(l);
    }
    const int M = (int)order.size(), ring = N - R;
    auto load = [&](int l, int s) {
        if (slot_layer_[s] >= 0) layer_slot_[slot_layer_[s]] = -1;
        slot_layer_[s] = l;
        layer_slot_[l] = s;
        fresh_[l] = 1;
        return sink.copy(l, s, slot_last_[s]);
    };
    if (dir > 0)
        for (int l = lo; l < R; ++l)
            if (layer_slot_[l] < 0 && (rc = load(l, l)) != SP_OK) return rc;
    // Initial load (Sec. 3.3: k partitions are on the device before the first compute):
    // the first `ring` streamed layers of the pass, except those still resident from the
    // previous pass.
    const int first = std::min(ring, M);
    std::vector<char> keep(N, 0);
    for (int i = 0; i < first; ++i)
        if (layer_slot_[order[i]] >= 0) keep[layer_slot_[order[i]]] = 1;
    int scan = R;
    for (int i = 0; i < first; ++i) {
        const int l = order[i];
        if (layer_slot_[l] >= 0) continue;
        while (scan < N && keep[scan]) ++scan;
        if (scan >= N) return SP_ERR_STATE;  // cannot happen: first <= ring
        keep[scan] = 1;
        if ((rc = load(l, scan)) != SP_OK) return rc;
    }
    if (dir < 0)
        for (int l = R - 1; l >= lo; --l)
            if (layer_slot_[l] < 0 && (rc = load(l, l)) != SP_OK) return rc;
    // Steady state (Sec. 3.3, Fig. 1): after each group of `group_` executed streamed
    // layers, their slots are refilled with the next streamed layers of the pass.
    int next = first;          // position in `order` of the next layer to fetch
    int wrapped = 0;           // streamed layers of the NEXT pass already fetched (wrap)
    int gbegin = 0;            // first position in `order` of the current group
    int mi = 0;                // streamed layers computed so far
    for (int i = 0; i < L; ++i) {
        const int l = dir > 0 ? i : L - 1 - i;
        if (l < lo) continue;
        const int s = layer_slot_[l];
        if (s < 0) return SP_ERR_STATE;
        if ((rc = sink.compute(l, s, dir, fresh_[l] != 0)) != SP_OK) return rc;
        fresh_[l] = 0;
        slot_last_[s] = l;
        if (l < R) continue;
        ++mi;
        if (mi - gbegin == group_ || mi == M) {
            for (int j = gbegin; j < mi; ++j) {
                const int done = order[j];
                int t = -1;
                while (next < M && layer_slot_[order[next]] >= 0) ++next;  // already on the device
                if (next < M) {
                    t = order[next++];
                } else if (wrap && ring < M) {
                    while (wrapped < ring && layer_slot_[order[wrapped]] >= 0) ++wrapped;
                    if (wrapped < ring) t = order[wrapped++];
                }
                if (t < 0) break;
                const int sl = layer_slot_[done];
                layer_slot_[done] = -1;
                slot_layer_[sl] = t;
                layer_slot_[t] = sl;
                fresh_[t] = 1;
                if ((rc = sink.copy(t, sl, done)) != SP_OK) return rc;
            }
            gbegin = mi;
        }
    }
    return SP_OK;
}

}  // namespace sp

// ---- host-only C entry points ---------------------------------------------------
using namespace sp;

extern "C" int sp_num_tensors(const sp_stack_desc* desc) {
    Layout lay;
    int rc = make_layout(desc, &lay);
    return rc == SP_OK ? lay.n_tensors : rc;
}

extern "C" size_t sp_tensor_offset(const sp_stack_desc* desc, int tensor_id) {
    Layout lay;
    if (make_layout(desc, &lay) != SP_OK || tensor_id < 0 || tensor_id >= lay.n_tensors) return (size_t)-1;
    return lay.t[tensor_id].offset;
}

extern "C" size_t sp_tensor_elems(const sp_stack_desc* desc, int tensor_id) {
    Layout lay;
    if (make_layout(desc, &lay) != SP_OK || tensor_id < 0 || tensor_id >= lay.n_tensors) return 0;
    return lay.t[tensor_id].elems;
}

extern "C" size_t sp_layer_blob_bytes(const sp_stack_desc* desc) {
    Layout lay;
    return make_layout(desc, &lay) == SP_OK ? lay.blob_bytes : 0;
}

extern "C" size_t sp_layer_grad_bytes(const sp_stack_desc* desc) {
    Layout lay;
    return make_layout(desc, &lay) == SP_OK ? lay.grad_bytes : 0;
}

extern "C" size_t sp_workspace_bytes(const sp_stack_desc* desc, int training) {
    Layout lay;
    if (make_layout(desc, &lay) != SP_OK) return 0;
    Workspace ws;
    make_workspace(desc, lay, training, &ws);
    return ws.total;
}

extern "C" int sp_make_plan(const sp_stack_desc* desc, int k, int p, int pinned_layers, uint64_t budget_bytes,
                            int training, sp_plan* out) {
    return make_plan(desc, 1, k, p, pinned_layers, budget_bytes, training, out);
}

extern "C" int sp_make_plan_units(const sp_stack_desc* desc, int units_per_layer, int k, int p, int pinned_units,
                                  uint64_t budget_bytes, int training, sp_plan* out) {
    return make_plan(desc, units_per_layer, k, p, pinned_units, budget_bytes, training, out);
}

extern "C" int sp_unit_range(const sp_stack_desc* desc, int units_per_layer, int part, uint64_t* offset,
                             uint64_t* bytes) {
    Layout lay;
    if (!offset || !bytes) return SP_ERR_INVALID_ARG;
    int rc = make_layout(desc, &lay);
    if (rc != SP_OK) return rc;
    size_t off = 0, len = 0;
    rc = unit_range(desc, lay, units_per_layer, part, &off, &len);
    if (rc != SP_OK) return rc;
    *offset = off;
    *bytes = len;
    return SP_OK;
}

namespace {
struct TraceSink : SchedSink {
    sp_sched_op* ops;
    int cap, n = 0, pass = 0;
    void push(int kind, int layer, int slot, int w) {
        if (n < cap) ops[n] = sp_sched_op{kind, layer, slot, w, pass};
        ++n;
    }
    int copy(int layer, int slot, int wait_layer) override { push(0, layer, slot, wait_layer); return SP_OK; }
    int compute(int layer, int slot, int dir, bool fresh) override { push(dir > 0 ? 1 : 2, layer, slot, fresh ? 1 : 0); return SP_OK; }
};
}  // namespace

static int trace_schedule(int n_layers, int n_slots, int n_pinned, int p_eff, int training, int wrap_prefetch,
                          int passes, const int* updated, int n_updated, sp_sched_op* ops, int cap) {
    // training > 1: backward passes stop after layer training - 1 (layers below are frozen)
    const int bwd_lo = training > 1 ? training - 1 : 0;
    if (n_layers < 1 || n_slots < 1 || n_slots > n_layers || n_pinned < 0 || n_pinned >= n_slots || p_eff < 1 ||
        passes < 1 || cap < 0 || (cap && !ops) || training < 0 || bwd_lo > n_layers || n_updated < 0 ||
        (n_updated && !updated))
        return SP_ERR_INVALID_ARG;
    for (int i = 0; i < n_updated; ++i)
        if (updated[i] < 0 || updated[i] >= n_layers) return SP_ERR_INVALID_ARG;
    Scheduler sch;
    sch.reset(n_layers, n_slots, p_eff, n_pinned);
    TraceSink sink;
    sink.ops = ops;
    sink.cap = cap;
    for (int ps = 0; ps < passes; ++ps) {
        sink.pass = ps;
        const int dir = (training && (ps & 1)) ? -1 : +1;
        if (dir > 0 && ps > 0)
            for (int i = 0; i < n_updated; ++i) sch.invalidate(updated[i]);
        int rc = sch.run_pass(dir, !training && wrap_prefetch, sink, dir < 0 ? bwd_lo : 0);
        if (rc != SP_OK) return rc;
    }
    return sink.n;
}

extern "C" int sp_trace_schedule(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                                 int wrap_prefetch, int passes, sp_sched_op* ops, int cap) {
    return trace_schedule(n_layers, n_slots, n_pinned, p_eff, training, wrap_prefetch, passes, nullptr, 0, ops, cap);
}

extern "C" int sp_trace_schedule_updated(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                                         int wrap_prefetch, int passes, const int* updated_layers, int n_updated,
                                         sp_sched_op* ops, int cap) {
    return trace_schedule(n_layers, n_slots, n_pinned, p_eff, training, wrap_prefetch, passes, updated_layers,
                          n_updated, ops, cap);
}

// ---- schedule cost model and window tuner ----------------------------------
namespace {
// Measured on MI355X: what one more copy / one more fenced compute operation costs when a layer
// is cut into units (llama7b: 87 instead of 30 copies per pass, +1.4 ms; ViT-H: 96 instead of 32
// computes, +4.3 ms).
constexpr double kCopyFixedMs = 0.025, kComputeFixedMs = 0.06;

// Plays the scheduler's decisions on three in-order streams (copy, compute, gradient
// copy) with fixed per-layer durations; the same dependencies the engine expresses as
// events become max() of end times here.
struct SimSink : SchedSink {
    const sp_layer_cost& c;
    // units > 1: op `layer` is unit q = layer % units of a layer; its copy takes the unit's share
    // of the bytes, its compute the unit's share of the layer's time, each plus a fixed cost per
    // extra operation (launch of a copy; the event wait in front of a compute)
    int units = 1;
    double copy_part[3] = {1, 0, 0}, fwd_part[3] = {1, 0, 0};
    double copy_ms_of(int layer) const {
        return units == 1 ? c.copy_ms : std::max(0.0, c.copy_ms - kCopyFixedMs) * copy_part[layer % units] + kCopyFixedMs;
    }
    double fwd_ms_of(int layer) const {
        return units == 1 ? c.fwd_ms : c.fwd_ms * fwd_part[layer % units] + kComputeFixedMs;
    }
    std::vector<double> loaded, done;
    double t_copy = 0, t_comp = 0, t_grad = 0, t_floor = 0;
    double gslot_free[kGradSlots] = {};
    int gs = 0;
    bool training = false;
    SimSink(const sp_layer_cost& cost, int L) : c(cost), loaded(L, 0.0), done(L, 0.0) {}
    int copy(int layer, int, int wait_layer) override {
        double b = std::max(t_copy, t_floor);
        if (wait_layer >= 0) b = std::max(b, done[wait_layer]);
        t_copy = b + copy_ms_of(layer);
        loaded[layer] = t_copy;
        return SP_OK;
    }
    int compute(int layer, int, int dir, bool fresh) override {
        double b = std::max(t_comp, t_floor);
        if (fresh) b = std::max(b, loaded[layer]);
        if (dir > 0) {
            t_comp = b + fwd_ms_of(layer);
        } else {
            b = std::max(b, gslot_free[gs]);            // its gradient slot must have drained
            t_comp = b + c.bwd_ms;
            t_grad = std::max(t_grad, t_comp) + c.grad_ms;
            gslot_free[gs] = t_grad;
            gs = (gs + 1) % kGradSlots;
        }
        done[layer] = t_comp;
        return SP_OK;
    }
    double now() const { return std::max(std::max(t_copy, t_comp), t_grad); }
};

double simulate(int L, int n_slots, int n_pinned, int p_eff, int training, int wrap, int calls,
                const sp_layer_cost& c, int units = 1, const double* copy_part = nullptr,
                const double* fwd_part = nullptr) {
    Scheduler sch;
    sch.reset(L, n_slots, p_eff, n_pinned);
    SimSink sink(c, L);
    sink.units = units;
    for (int q = 0; q < units && units > 1; ++q) { sink.copy_part[q] = copy_part[q]; sink.fwd_part[q] = fwd_part[q]; }
    double begin = 0, end = 0;
    for (int i = 0; i < calls; ++i) {
        // forward-only calls follow each other on the streams; a training step starts
        // when the previous one has delivered its last gradient
        begin = training ? sink.now() : sink.t_comp;
        if (training) sink.t_floor = begin;
        sch.run_pass(+1, !training && wrap, sink);
        if (training) sch.run_pass(-1, false, sink);
        end = training ? sink.now() : sink.t_comp;
    }
    return end - begin;
}
}  // namespace

extern "C" double sp_simulate_call_ms(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                                      int wrap_prefetch, int calls, const sp_layer_cost* cost) {
    if (n_layers < 1 || n_slots < 1 || n_slots > n_layers || n_pinned < 0 || n_pinned >= n_slots || p_eff < 1 ||
        calls < 1 || !cost ||
        !(cost->copy_ms >= 0) || !(cost->fwd_ms >= 0) || !(cost->bwd_ms >= 0) || !(cost->grad_ms >= 0))
        return -1.0;
    return simulate(n_layers, n_slots, n_pinned, p_eff, training, wrap_prefetch, calls, *cost);
}

extern "C" int sp_autotune(const sp_stack_desc* desc, uint64_t budget_bytes, int training, int wrap_prefetch,
                           const sp_layer_cost* cost, double tolerance, int* k_out, int* p_out, int* pinned_out,
                           double* ms_out) {
    const char* why = nullptr;
    if (!desc || !cost || !k_out || !p_out || !pinned_out || validate_desc(desc, &why) != SP_OK || !(tolerance >= 0))
        return SP_ERR_INVALID_ARG;
    const int L = desc->n_layers;
    struct Cand { int n, r, p; double ms; };
    std::vector<Cand> cands;
    int rc_first = SP_OK;
    // windows without pinned layers, and the same windows with the rest of the budget pinned
    for (int pin = 0; pin < 2; ++pin) {
        for (int p = 1; p <= L; ++p) {
            for (int k = 1; k + p <= L + 1; ++k) {
                sp_plan pl;
                int rc = make_plan(desc, 1, k, p, pin ? SP_PIN_AUTO : 0, budget_bytes, training, &pl);
                if (rc != SP_OK) { if (rc_first == SP_OK) rc_first = rc; continue; }
                bool seen = false;
                for (const Cand& c : cands) seen = seen || (c.n == pl.n_slots && c.r == pl.n_pinned && c.p == pl.p_eff);
                if (seen) continue;
                const double ms = sp_simulate_call_ms(L, pl.n_slots, pl.n_pinned, pl.p_eff, training ? 1 : 0,
                                                      wrap_prefetch, 3, cost);
                if (ms < 0) return SP_ERR_INVALID_ARG;
                cands.push_back(Cand{pl.n_slots, pl.n_pinned, pl.p_eff, ms});
            }
        }
    }
    if (cands.empty()) return rc_first != SP_OK ? rc_first : SP_ERR_BUDGET;
    double best = cands[0].ms;
    for (const Cand& c : cands) best = std::min(best, c.ms);
    const Cand* pick = nullptr;
    for (const Cand& c : cands) {
        if (c.ms > best * (1.0 + tolerance)) continue;
        if (!pick || c.n < pick->n || (c.n == pick->n && c.p < pick->p)) pick = &c;
    }
    *p_out = pick->p;
    *k_out = std::max(pick->n - pick->r - pick->p, 1);
    *pinned_out = pick->r;
    if (ms_out) *ms_out = pick->ms;
    return SP_OK;
}

// Shares of a layer's bytes and of its arithmetic that fall to each of the three units.
static void unit_shares(const sp_stack_desc* d, const Layout& lay, double* copy_part, double* fwd_part) {
    double flops[3];
    const double T = 1.0, dm = d->d_model, f = d->d_ffn;
    const double nq = (double)d->n_q_heads * d->head_dim, nkv = (double)d->n_kv_heads * d->head_dim;
    const double S = d->max_seq;
    flops[0] = 2 * T * dm * (nq + 2 * nkv) + 2 * T * nq * dm + 4 * T * S * nq * (d->causal ? 0.5 : 1.0);
    flops[1] = 2 * T * dm * f * (d->arch == SP_DECODER_SWIGLU_RMS ? 2 : 1);
    flops[2] = 2 * T * f * dm;
    const double fsum = flops[0] + flops[1] + flops[2];
    for (int q = 0; q < 3; ++q) {
        size_t off, len;
        unit_range(d, lay, 3, q, &off, &len);
        copy_part[q] = (double)len / (double)lay.blob_bytes;
        fwd_part[q] = flops[q] / fsum;
    }
}

extern "C" int sp_autotune_units(const sp_stack_desc* desc, uint64_t budget_bytes, int training, int wrap_prefetch,
                                 const sp_layer_cost* cost, double tolerance, int* units_out, int* k_out, int* p_out,
                                 int* pinned_out, double* ms_out) {
    if (!units_out) return SP_ERR_INVALID_ARG;
    double ms1 = 0;
    int rc = sp_autotune(desc, budget_bytes, training, wrap_prefetch, cost, tolerance, k_out, p_out, pinned_out, &ms1);
    if (rc != SP_OK) return rc;
    *units_out = 1;
    if (ms_out) *ms_out = ms1;
    if (training) return SP_OK;
    Layout lay;
    make_layout(desc, &lay);
    double copy_part[3], fwd_part[3];
    unit_shares(desc, lay, copy_part, fwd_part);
    const int L = desc->n_layers * 3;
    // in units only the smallest windows are of interest: what a larger one buys is bought more
    // cheaply by pinning, which is what the rest of the budget does
    double best = -1;
    int bk = 0, bp = 0, br = 0;
    for (int p = 1; p <= 2; ++p)
        for (int k = 1; k <= 2; ++k) {
            sp_plan pl;
            if (make_plan(desc, 3, k, p, SP_PIN_AUTO, budget_bytes, 0, &pl) != SP_OK) continue;
            if (pl.n_pinned >= pl.n_slots || pl.n_slots > L) continue;
            const double ms = simulate(L, pl.n_slots, pl.n_pinned, pl.p_eff, 0, wrap_prefetch, 3, *cost, 3, copy_part,
                                       fwd_part);
            if (best < 0 || ms < best) { best = ms; bk = pl.k_eff; bp = pl.p_eff; br = pl.n_pinned; }
        }
    if (best >= 0 && best < ms1 * (1.0 - tolerance)) {      // worth the extra fences only when clearly faster
        *units_out = 3; *k_out = bk; *p_out = bp; *pinned_out = br;
        if (ms_out) *ms_out = best;
    }
    return SP_OK;
}
