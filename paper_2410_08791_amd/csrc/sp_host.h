// Host-side logic shared by the engine and the layout/plan queries:
// blob layout, workspace carving, slot-count policy and the window scheduler.
// Pure C++ (no HIP calls) so that it can be exercised without a device.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/superpipe.h"

namespace sp {

constexpr size_t kTensorAlign = 256;
constexpr size_t kSlotAlign = 4096;
constexpr int kMaxTensors = 12;
constexpr int kGradSlots = 4;   // fp32 gradient slots cycled by the backward pass

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct TensorInfo {
    size_t offset;  // bytes inside the bf16 weight blob
    size_t elems;
    int rows, cols;  // vectors: rows = 1
};

struct Layout {
    int n_tensors = 0;
    TensorInfo t[kMaxTensors];
    size_t blob_bytes = 0;   // bf16 weights
    size_t grad_bytes = 0;   // fp32 gradients: offsets doubled
};

// Returns SP_OK or SP_ERR_INVALID_ARG (why: optional text).
int validate_desc(const sp_stack_desc* d, const char** why);
int make_layout(const sp_stack_desc* d, Layout* out);

// Device workspace, as byte offsets from its base (all 256-byte aligned).
struct Workspace {
    size_t a, qkv, o, gu, z;               // forward activations (bf16)
    size_t set_stride;                     // > 0: layer l's copy of {a,qkv,o,gu,z,m,h1,lse} lies l*set_stride further
    // training only
    size_t xs;                             // layer inputs fp32 [L][T, d], kept for the backward
    size_t m;                              // second normed activation bf16 [Tp, d]
    size_t h1;                             // residual after attention fp32 [T, d]
    size_t lse, delta;                     // softmax log-sum-exp, rowsum(dO*O): fp32 [B, Hq, S]
    size_t dh, da;                         // fp32 [T, d]: stream gradient, norm-output gradient
    size_t dhb;                            // bf16 [Tp, d] copy of dh (GEMM operand)
    size_t dqkv, dob, dz;                  // bf16 gradients of qkv, attention output, SwiGLU output
    size_t part;                           // fp32 [kNormBwdBlocks, d] gain-gradient partials (+ loss partials)
    size_t gslot[kGradSlots];              // fp32 gradient slots
    size_t total;
    int t_pad;                             // token rows padded to 64 (training)
};
// training: 0 = forward only, 1 = training with per-layer recompute, 2 = training keeping every
// layer's activations (no recompute)
void make_workspace(const sp_stack_desc* d, const Layout& lay, int training, Workspace* ws);

// Byte range of part `part` of a layer blob when a layer streams as `units` units (1 or 3).
int unit_range(const sp_stack_desc* d, const Layout& lay, int units, int part, size_t* off, size_t* len);
int make_plan(const sp_stack_desc* d, int units, int k, int p, int pinned, uint64_t budget, int training, sp_plan* out);

// ---- window scheduler --------------------------------------------------------
// Decides, in host order, which layer is copied into which slot and when a
// slot may be reused; the engine turns each decision into stream operations,
// the tracer records them.  Residency survives across passes.
struct SchedSink {
    virtual ~SchedSink() {}
    // copy `layer` into `slot`; it must start after the compute of `wait_layer` (-1: none)
    virtual int copy(int layer, int slot, int wait_layer) = 0;
    // run `layer` (dir +1 forward, -1 backward) out of `slot`
    virtual int compute(int layer, int slot, int dir, bool copied_since_last_use) = 0;
};

class Scheduler {
public:
    // n_pinned: layers 0..n_pinned-1 keep a slot each for good; the others stream through the rest
    void reset(int n_layers, int n_slots, int group, int n_pinned = 0);
    // One pass over all layers: dir +1 = 0..L-1, dir -1 = L-1..0.  With wrap
    // (forward-only use) slots freed at the tail are refilled with the first layers.
    // lo: the pass covers layers lo..L-1 only (a backward pass that stops above frozen layers).
    int run_pass(int dir, bool wrap, SchedSink& sink, int lo = 0);
    // The caller rewrote `layer`'s host copy: forget the device copy, the next pass fetches it again.
    // The slot remembers its last user, so the new copy still waits for that compute.
    void invalidate(int layer);
    int n_slots() const { return n_slots_; }
    int n_pinned() const { return n_pinned_; }
    const std::vector<int>& layer_slot() const { return layer_slot_; }

private:
    int n_layers_ = 0, n_slots_ = 0, group_ = 1, n_pinned_ = 0;
    std::vector<int> slot_layer_;   // layer occupying (or being copied into) a slot, -1 = empty
    std::vector<int> slot_last_;    // last layer computed out of a slot, -1 = none
    std::vector<int> layer_slot_;   // slot of a resident layer, -1 = not on the device
    std::vector<char> fresh_;       // copied since last compute
};

}  // namespace sp
