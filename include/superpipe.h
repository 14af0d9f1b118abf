/*
 * superpipe.h -- C ABI of the MI355X layer-streaming executor.
 *
 * The library runs a stack of identical transformer layers whose bf16 weights
 * live in pinned host memory.  Only a window of layers is resident in HBM; the
 * next layers are copied host-to-device on a side stream while the resident
 * ones compute, and a layer's slot is overwritten once it has executed.  This
 * is the Superpipeline schedule (paper Sec. 1, Fig. 1; Sec. 3.2.2; Sec. 3.3):
 * partitions = repeated layers (Sec. 3.2.1), k partitions on the device, k'
 * swapped per group, forward and backward (Sec. 3.3), with results identical
 * to the fully resident run (Sec. 4.2).  Copying weights back to the host is
 * replaced by overwriting the slot, the design the paper's Sec. 5 proposes.
 *
 * Conventions
 *  - Every call returns SP_OK (0) or a negative sp_status; nothing aborts or
 *    throws across the boundary.  sp_last_error() gives a text for the most
 *    recent failure on a handle (or of sp_create when passed NULL).
 *  - "host" pointers are CPU addresses, "dev" pointers are HBM addresses on
 *    the current HIP device.  The library allocates NO device memory: slots
 *    and workspace are carved from the caller's arena, so peak HBM use is
 *    arena_bytes_used <= gpu_budget_bytes by construction.
 *  - Calls enqueue work and return; outputs are valid after the caller
 *    synchronises compute_stream (gradient blobs: d2h_stream).  Three places
 *    block the host, none for longer than the work already enqueued: (1) the
 *    run-ahead bound -- when about 1400 kernel launches and event records of a
 *    handle are still unfinished on its compute stream, the next layer's enqueue
 *    waits until about 350 are left (every call kind; a deep stack reaches the
 *    bound inside one call; beyond it this HIP runtime was measured to run whole
 *    passes 30-60 % slower); (2) sp_forward_backward waits at entry for the
 *    previous step's last gradient; (3) sp_wait_gradient, sp_get_stats with a
 *    timing flag, and sp_destroy wait for what they name.
 *  - Kernel and tile choice depend on the shapes in sp_stack_desc and on B, S only:
 *    never on the window, the slot address or the process environment (the library
 *    reads no environment variable).
 *  - One handle = one stack; calls on a handle must not overlap.  Handles may be
 *    used from different host threads, one thread at a time per handle.
 *  - A call that fails after it has begun to enqueue a pass (SP_ERR_HIP from a copy,
 *    launch or event call mid-pass) leaves the handle FAILED: slots may hold layers
 *    whose copies were never issued, so every later call on it returns SP_ERR_STATE;
 *    sp_last_error and sp_destroy keep working.  Argument errors (INVALID_ARG, SHAPE,
 *    NOT_PINNED, STATE) are detected before anything is enqueued and leave the handle usable.
 */
#ifndef SUPERPIPE_H
#define SUPERPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sp_engine* sp_handle;

typedef enum {
    SP_OK = 0,
    SP_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, bad enum, bad struct_size */
    SP_ERR_BUDGET = -2,      /* arena cannot hold the workspace plus one layer slot          */
    SP_ERR_NOT_PINNED = -3,  /* a host blob is not page-locked host memory                   */
    SP_ERR_HIP = -4,         /* a HIP runtime call failed; see sp_last_error                 */
    SP_ERR_STATE = -5,       /* handle destroyed / created forward-only but asked to train   */
    SP_ERR_SHAPE = -6        /* B or S outside what the workspace was sized for              */
} sp_status;

/* Layer kinds.  Decoder: pre-RMSNorm, fused QKV, SwiGLU FFN, no biases.
 * Encoder: pre-LayerNorm (gain+bias), biased projections, exact-erf GELU MLP. */
enum { SP_DECODER_SWIGLU_RMS = 0, SP_ENCODER_GELU_LN = 1 };

/* Tensors of one layer, in blob order.  Matrices are row-major [out, in]
 * (y = x W^T), bf16.  WQKV stacks query rows, key rows, value rows; WGU stacks
 * gate rows then up rows.  Every tensor starts on a 256-byte boundary. */
enum {
    /* decoder */
    SP_T_G1 = 0, SP_T_WQKV = 1, SP_T_WO = 2, SP_T_G2 = 3, SP_T_WGU = 4, SP_T_WD = 5,
    SP_DECODER_TENSORS = 6,
    /* encoder */
    SP_T_LN1_G = 0, SP_T_LN1_B = 1, SP_T_E_WQKV = 2, SP_T_BQKV = 3, SP_T_E_WO = 4, SP_T_BO = 5,
    SP_T_LN2_G = 6, SP_T_LN2_B = 7, SP_T_W1 = 8, SP_T_B1 = 9, SP_T_W2 = 10, SP_T_B2 = 11,
    SP_ENCODER_TENSORS = 12
};

typedef struct {
    uint32_t struct_size;   /* = sizeof(sp_stack_desc) */
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;     /* divides n_q_heads; query head j uses kv head j / (n_q/n_kv) */
    int32_t head_dim;       /* 64, 80 or 128 */
    int32_t d_ffn;
    int32_t arch;           /* SP_DECODER_SWIGLU_RMS | SP_ENCODER_GELU_LN */
    int32_t causal;         /* 1: query i attends keys j <= i */
    float norm_eps;
    int32_t max_batch;      /* workspace is sized for max_batch * max_seq tokens */
    int32_t max_seq;
} sp_stack_desc;

enum {
    SP_FLAG_TRAINING = 1u << 0,    /* size the workspace for sp_forward_backward           */
    SP_FLAG_TIMING = 1u << 1,      /* record per-layer copy/compute events (sp_get_stats)  */
    SP_FLAG_POISON = 1u << 2,      /* debug: fill a slot with NaN patterns before reuse    */
    SP_FLAG_NO_OVERLAP = 1u << 3,  /* "Naive" comparator (Sec. 4.2): copies wait for all
                                      enqueued compute, compute waits for the copies       */
    SP_FLAG_WRAP_PREFETCH = 1u << 4, /* forward-only: when the tail of a pass frees slots,
                                      start loading layers 0.. for the next call (the
                                      consecutive-forward stall of Sec. 5)                 */
    SP_FLAG_KEEP_ACTIVATIONS = 1u << 6, /* training: keep every layer's activations in the
                                      workspace instead of recomputing them in the backward
                                      (the columns of Table 2 that train without gradient
                                      checkpointing): more HBM, about a quarter less compute */
    SP_FLAG_KERNEL_TIMING = 1u << 5, /* bracket every 4th launch of the layer's largest GEMM with
                                      timed events on the compute stream (big_gemm_* in sp_stats) */
    SP_FLAG_OP_TIMING = 1u << 8,   /* bracket EVERY kernel launch of the layers with timed events on the compute
                                      stream and sum the durations per operation kind (op_ms / op_launches in
                                      sp_stats).  The event records leave gaps on the stream, so a pass runs
                                      slower than without the flag; the per-kernel durations are what it is for */
    SP_FLAG_DELAY = 1u << 7        /* debug: pseudo-random delays of up to sp_config.delay_us each -- the
                                      host sleeps between enqueues, and a one-wave kernel that idles for a
                                      bounded time and exits runs in front of every layer copy (copy stream)
                                      and every layer's kernels (compute stream).  The streams then drift
                                      against each other in ways a fast run never shows; a missing fence
                                      surfaces as changed output bits (with SP_FLAG_POISON: as NaN).
                                      Results must not change (Sec. 4.2)                              */
};

typedef struct {
    uint32_t struct_size;       /* = sizeof(sp_config) */
    int32_t resident_window_k;  /* layers kept ready to compute            (>= 1) */
    int32_t prefetch_depth_p;   /* layers in flight / swapped per group    (>= 1) */
    uint64_t gpu_budget_bytes;  /* size of device_arena; the hard HBM cap        */
    void* device_arena;         /* dev, caller-owned, 4 KiB aligned              */
    void* compute_stream;       /* hipStream_t (NULL = default stream)           */
    void* h2d_stream;           /* hipStream_t, must differ from compute_stream  */
    void* d2h_stream;           /* hipStream_t, needed only with SP_FLAG_TRAINING */
    uint32_t flags;
    int32_t frozen_layers;      /* training: layers 0..n-1 receive no weight gradients (the rows
                                   of Table 2 with half of the layers frozen).  Their gradient
                                   blobs are not written; when sp_forward_backward is called with
                                   dx_dev == NULL the backward pass stops above them, so they
                                   are neither re-streamed nor recomputed.                     */
    int32_t pinned_layers;      /* layers 0..n-1 that stay in HBM for the handle's life and are
                                   never re-copied; SP_PIN_AUTO = as many as the budget leaves
                                   after the k + p window; 0 = none (every layer streams)      */
    int32_t units_per_layer;    /* 0 or 1: a layer is the unit that streams (the paper's partition at
                                   the repeated-layer boundaries, Sec. 3.2.1).  3: a layer streams as
                                   three units in blob order -- the attention block (first norm, QKV and
                                   output projections), the first FFN projection (second norm, gate/up or
                                   W1) and the last FFN projection (down or W2) -- and k, p,
                                   pinned_layers and every per-layer figure of sp_plan / sp_stats count
                                   UNITS.  The double buffer then costs two of the largest unit instead
                                   of two layers and the budget pins more of the stack (pinned units are
                                   stored at their own size).  Forward-only handles (no SP_FLAG_TRAINING);
                                   results are bit-identical to layer units.                            */
    int32_t delay_us;           /* SP_FLAG_DELAY: upper bound of one injected delay, 1..20000 microseconds
                                   (0 with the flag set = 200); ignored without the flag               */
} sp_config;
#define SP_PIN_AUTO (-1)

/* Slot-count policy (one function decides it).  The streaming window asks for
 * k + p HBM layer slots -- the paper's k (partitions held on the GPU) with its k' = p
 * of them being refilled (Fig. 1: k=4, k'=2 is (k,p) = (2,2)) -- clamped by the
 * layer count and by what the arena holds after the workspace; pinned layers
 * take what the budget leaves after the window:
 *   cap      = min(L, (budget - workspace) / slot_bytes);   0 -> SP_ERR_BUDGET
 *   window   = min(k + p, cap)
 *   n_pinned = min(pinned_layers, cap - window)   (SP_PIN_AUTO: cap - window)
 *   n_slots  = window + n_pinned;  if that reaches L: fully resident, n_pinned = 0
 *   p_eff    = min(p, max(window - 1, 1)),  k_eff = max(window - p_eff, 1).
 * With n_pinned layers held, a steady-state pass copies L - n_pinned blobs
 * instead of L: on a link-bound stack that is the only way to go faster at a
 * fixed budget once the link is saturated.
 * With units_per_layer = 3 the same policy runs over the 3 L units: slot_bytes is the
 * largest unit, the window takes k + p such slots, and the pinned units 0, 1, ... take
 * their own sizes while they fit (sp_make_plan_units). */
typedef struct {
    int32_t n_slots, k_eff, p_eff;
    int32_t fully_resident;     /* n_slots == number of units */
    uint64_t slot_bytes;        /* bytes of the largest unit (layer blob, or its largest part) rounded up to 4 KiB */
    uint64_t workspace_bytes;
    uint64_t arena_bytes_used;  /* workspace + pinned_bytes + (n_slots - n_pinned) * slot_bytes (+ gradient slots) */
    int32_t n_pinned;           /* of the n_slots, those holding units 0..n_pinned-1 for good */
    int32_t units_per_layer;    /* 1 or 3 */
    uint64_t pinned_bytes;      /* what the pinned units occupy: each its own size rounded up to 4 KiB */
} sp_plan;

#define SP_MAX_TRACE_LAYERS 256
/* Operation kinds of SP_FLAG_OP_TIMING. */
enum {
    SP_OP_NORM = 0,        /* RMSNorm / LayerNorm, forward (and the backward pass's recompute)          */
    SP_OP_GEMM_QKV = 1,    /* fused q/k/v projection                                                    */
    SP_OP_ATTENTION = 2,   /* attention forward (with a cache: append + single-query attention)         */
    SP_OP_GEMM_O = 3,      /* output projection + residual                                              */
    SP_OP_GEMM_FFN1 = 4,   /* gate/up (SwiGLU in the epilogue when forward-only) or first MLP projection */
    SP_OP_ACT = 5,         /* SwiGLU / GELU as a kernel of its own (training keeps the pre-activations) */
    SP_OP_GEMM_FFN2 = 6,   /* down / second MLP projection + residual                                   */
    SP_OP_LOSS = 7,        /* MSE loss and its gradient                                                 */
    SP_OP_GEMM_DW = 8,     /* the weight-gradient GEMMs (contraction over tokens)                       */
    SP_OP_GEMM_DX = 9,     /* the input-gradient GEMMs                                                  */
    SP_OP_ACT_BWD = 10,    /* SwiGLU / GELU backward                                                    */
    SP_OP_NORM_BWD = 11,   /* norm backward incl. its gain (and bias) gradient                          */
    SP_OP_ATTENTION_BWD = 12, /* rowsum(dO * O), dq kernel, dk/dv kernel                               */
    SP_OP_BIAS_GRAD = 13,  /* column sums for the bias gradients (encoder)                              */
    SP_OP_COPY = 14,       /* copies and fills of activations (x -> y, padded rows)                     */
    SP_N_OPS = 15
};
typedef struct {
    uint32_t struct_size;
    sp_plan plan;
    uint64_t calls;             /* completed sp_forward / sp_forward_backward calls   */
    uint64_t h2d_copies, h2d_bytes;   /* totals since create                            */
    uint64_t d2h_copies, d2h_bytes;
    uint64_t last_h2d_copies, last_h2d_bytes;  /* issued by the most recent call        */
    /* SP_FLAG_TIMING only; describe the most recent call, valid after its streams
     * are synchronised.  Times in ms relative to the call's first enqueued op.        */
    int32_t n_timed;                    /* entries below (forward layers, then backward) */
    float copy_begin_ms[SP_MAX_TRACE_LAYERS], copy_end_ms[SP_MAX_TRACE_LAYERS]; /* <0: no copy */
    float comp_begin_ms[SP_MAX_TRACE_LAYERS], comp_end_ms[SP_MAX_TRACE_LAYERS];
    float copy_busy_ms;         /* sum of copy durations                                */
    float copy_hidden_ms;       /* part of it that lies under some layer's compute      */
    float compute_busy_ms;      /* sum of layer compute durations                       */
    float wall_ms;              /* first op begin -> last op end                        */
    /* SP_FLAG_KERNEL_TIMING (or SP_FLAG_TIMING): the layer's largest GEMM (decoder: gate/up with the SwiGLU
     * epilogue; encoder: the first MLP GEMM), bracketed by events on the compute
     * stream at every 4th launch since the previous sp_get_stats (a sample: each pair
     * of event records leaves a gap on the stream).                                   */
    uint32_t big_gemm_launches;
    float big_gemm_ms_sum;
    int32_t big_gemm_m, big_gemm_n, big_gemm_k;   /* its shape: C[m,n] over k (n counts gate and up) */
    /* SP_FLAG_OP_TIMING: per operation kind (SP_OP_*), summed over the calls since the previous
     * sp_get_stats: total duration and number of launches. */
    float op_ms[16];
    uint32_t op_launches[16];
    int32_t n_ops;              /* SP_FLAG_TIMING: compute operations the most recent call issued (units, forward
                                   then backward); the arrays above hold the first n_timed = min(n_ops,
                                   SP_MAX_TRACE_LAYERS) of them, the busy/hidden/wall sums cover all n_ops */
} sp_stats;

/* ---- layout queries (host only, no device needed) ------------------------ */

/* Number of tensors per layer for desc->arch, or a negative sp_status. */
int sp_num_tensors(const sp_stack_desc* desc);
/* Byte offset of tensor `tensor_id` inside a layer blob; (size_t)-1 on bad args. */
size_t sp_tensor_offset(const sp_stack_desc* desc, int tensor_id);
/* Element count of tensor `tensor_id` (bf16 elements); 0 on bad args. */
size_t sp_tensor_elems(const sp_stack_desc* desc, int tensor_id);
/* Bytes of one layer's weight blob (bf16).  0 on bad args. */
size_t sp_layer_blob_bytes(const sp_stack_desc* desc);
/* Bytes of one layer's fp32 gradient blob: same tensor order, offsets doubled. */
size_t sp_layer_grad_bytes(const sp_stack_desc* desc);
/* Device workspace for max_batch*max_seq tokens.  training: 0 = forward only; 1 = training
 * (saved layer inputs, backward scratch, gradient slots); 2 = training with
 * SP_FLAG_KEEP_ACTIVATIONS (one activation set per layer). */
size_t sp_workspace_bytes(const sp_stack_desc* desc, int training);
/* The slot-count policy above as a pure function (layer units). */
int sp_make_plan(const sp_stack_desc* desc, int k, int p, int pinned_layers, uint64_t budget_bytes,
                 int training, sp_plan* out);
/* The same with units_per_layer in {1, 3} (k, p, pinned in units).  With 3 the pinned units take
 * their own sizes: the window's k + p slots of the largest unit come first, then units 0, 1, ... are
 * pinned while they fit; the stack counts as fully resident only if every unit fits a slot of the
 * largest unit's size, otherwise at least one unit keeps streaming. */
int sp_make_plan_units(const sp_stack_desc* desc, int units_per_layer, int k, int p, int pinned_units,
                       uint64_t budget_bytes, int training, sp_plan* out);
/* Byte range of part `part` (0 .. units_per_layer-1) inside a layer blob. */
int sp_unit_range(const sp_stack_desc* desc, int units_per_layer, int part, uint64_t* offset, uint64_t* bytes);

/* One step of the host-side schedule, for inspection and host-only tests.
 * sp_trace_schedule writes the ordered op list that `passes` consecutive calls
 * would enqueue (dir +1 = forward pass over layers 0..L-1, the pattern
 * forward,backward repeats when training != 0).  Returns the number of ops
 * (may exceed cap; only cap are written) or a negative sp_status.  n_slots
 * counts every slot, the n_pinned < n_slots pinned ones included.  training = 1 + F
 * traces backward passes that stop above F frozen layers (layers F..L-1 only). */
typedef struct {
    int32_t kind;    /* 0 = COPY layer->slot (copy stream), 1 = COMPUTE layer (compute stream),
                        2 = BACKWARD layer (compute stream) */
    int32_t layer, slot;
    int32_t wait_layer;  /* COPY: the layer whose compute must finish first (-1 none);
                            COMPUTE/BACKWARD: 1 if it waits for a copy issued earlier, else 0 */
    int32_t pass;
} sp_sched_op;
int sp_trace_schedule(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                      int wrap_prefetch, int passes, sp_sched_op* ops, int cap);
/* The same with the caller rewriting host weights between calls: before every forward
 * pass but the first, sp_weights_updated is applied to each of updated_layers[0..n_updated-1]
 * (host, may be NULL when n_updated = 0). */
int sp_trace_schedule_updated(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                              int wrap_prefetch, int passes, const int* updated_layers, int n_updated,
                              sp_sched_op* ops, int cap);

/* Cost model of the schedule (host only).  Plays what sp_trace_schedule lists on
 * three in-order streams -- layer copies, layer computes, gradient copies --
 * with one duration per kind, and returns the duration in ms of the last of
 * `calls` consecutive calls (forward passes, or training steps when training != 0;
 * a training step starts when the previous one has delivered its gradients).
 * Durations come from a measurement (sp_stats' per-layer trace) or from
 * bytes / link rate and FLOP / rate.  Returns < 0 on invalid arguments. */
typedef struct {
    double copy_ms;   /* one layer blob, host to device             */
    double fwd_ms;    /* one layer forward (training: incl. what the forward pass does) */
    double bwd_ms;    /* one layer backward incl. recompute (training only)             */
    double grad_ms;   /* one layer's gradient copy, device to host (training only)      */
} sp_layer_cost;
double sp_simulate_call_ms(int n_layers, int n_slots, int n_pinned, int p_eff, int training,
                           int wrap_prefetch, int calls, const sp_layer_cost* cost);

/* Window choice under a byte budget (the paper finds k and k' by grid search,
 * Sec. 4.2, and names adaptive selection as future work, Sec. 5): every (k, p)
 * whose plan fits budget_bytes, once with no pinned layers and once with the
 * rest of the budget pinned, is run through the cost model; of those within
 * (1 + tolerance) of the best modelled time the one with the fewest slots, then
 * the smallest p, is returned (fewest bytes of HBM for the same speed).
 * training: 0, 1 or 2 as for sp_workspace_bytes.  SP_ERR_BUDGET if nothing fits. */
int sp_autotune(const sp_stack_desc* desc, uint64_t budget_bytes, int training, int wrap_prefetch,
                const sp_layer_cost* cost, double tolerance, int* k_out, int* p_out, int* pinned_out,
                double* ms_out);

/* The same choice with the unit size included: the layer-unit proposal of sp_autotune against
 * three units per layer (windows of 1..2 + 1..2 unit slots, the rest of the budget pinned).  A
 * unit's copy is charged its share of the layer's bytes, its compute its share of the layer's
 * arithmetic, each plus the measured fixed cost of one more copy / one more fenced compute
 * operation; units are proposed only when the modelled time is better by more than `tolerance`.
 * Training handles stream whole layers: *units_out = 1. */
int sp_autotune_units(const sp_stack_desc* desc, uint64_t budget_bytes, int training, int wrap_prefetch,
                      const sp_layer_cost* cost, double tolerance, int* units_out, int* k_out, int* p_out,
                      int* pinned_out, double* ms_out);

/* ---- the four calls ------------------------------------------------------ */

/* Create an executor.  layer_host_blobs[n_layers]: host, pinned, each
 * sp_layer_blob_bytes long, caller-owned, must stay valid until sp_destroy and
 * UNMODIFIED except as sp_weights_updated allows (the library never writes them:
 * the method leaves parameters untouched, Sec. 1).  Entries may alias.  On failure
 * *out is NULL. */
int sp_create(sp_handle* out, const sp_stack_desc* desc, const void* const* layer_host_blobs,
              const sp_config* cfg);

/* y = stack(x): one forward pass of the streamed stack (Sec. 3.3: the layers execute in order
 * while the window slides; Sec. 4.2: the result is that of the resident model).  Layers that are
 * not on the device are copied in as their slots free up, each layer is computed as soon as its
 * weights have landed.  x_dev, y_dev: dev, fp32 [B, S, d_model], may be the same buffer (y_dev
 * holds the residual stream while the pass runs).  1 <= B <= max_batch, 1 <= S <= max_seq
 * (SP_ERR_SHAPE otherwise); both 16-byte aligned.  Returns once the pass is enqueued. */
int sp_forward(sp_handle h, const float* x_dev, float* y_dev, int B, int S);

/* Autoregressive generation (the paper quotes its LLM results in ms per token,
 * Sec. 4.2, Table 1): every generated token is one pass over the streamed stack.
 * Causal decoder stacks with head_dim 64 or 128 only (SP_ERR_STATE otherwise).
 *
 * kv_cache_dev: dev, caller-owned, sp_kv_cache_bytes(desc, B, max_len) bytes, 16-byte
 * aligned, used with the same B and max_len in every call of one generation.  Per
 * layer it holds the keys transposed, bf16 [B][Hkv][head_dim][max_len], then the
 * values, bf16 [B][Hkv][max_len][head_dim].  max_len: multiple of 8, <= 32768.
 *
 * sp_prefill: y = stack(x) over S prompt positions per sequence (x_dev, y_dev: dev,
 * fp32 [B, S, d_model], as sp_forward) and stores their keys and values at cache
 * positions 0..S-1.
 * sp_decode: one new position per sequence.  x_dev, y_dev: dev, fp32 [B, d_model];
 * the token sits at position pos (the same for every sequence: pos positions are
 * already cached), its keys/values are stored at pos and its query attends to
 * positions 0..pos.  pos < max_len.
 * Both return once the pass is enqueued, like sp_forward. */
size_t sp_kv_cache_bytes(const sp_stack_desc* desc, int batch, int max_len);
int sp_prefill(sp_handle h, const float* x_dev, float* y_dev, void* kv_cache_dev, int B, int S, int max_len);
int sp_decode(sp_handle h, const float* x_dev, float* y_dev, void* kv_cache_dev, int B, int pos, int max_len);

/* One training step's device work (Sec. 3.3): forward, loss =
 * mean((y - target)^2), backward with each layer's weights re-streamed in
 * reverse order, fp32 weight gradients written (overwrite, not accumulate) to
 * grad_host_blobs[l] (host, pinned -- checked, SP_ERR_NOT_PINNED otherwise: from pageable
 * memory the gradient copies would block the host and lose their overlap with the backward
 * pass -- sp_layer_grad_bytes each) over d2h_stream.
 * loss_dev: dev, 1 fp32.  dx_dev: dev fp32 [B,S,d] or NULL.  y_dev may be NULL.
 * The call returns once the step is enqueued.  At most one training step is in
 * flight per handle: a call first blocks the host until the previous step's
 * last gradient has landed (the point its consumer, the host-side optimizer,
 * has to wait for anyway before the weights of the next step exist). */
int sp_forward_backward(sp_handle h, const float* x_dev, const float* target_dev, float* y_dev,
                        float* loss_dev, float* dx_dev, void* const* grad_host_blobs, int B, int S);

/* A training LOOP (Sec. 3.3 runs forward and backward over the same streamed layers;
 * between two steps the caller's optimizer rewrites the host weights).
 *
 * sp_wait_gradient blocks the host until `layer`'s gradient of the latest
 * sp_forward_backward has landed in its grad_host_blobs entry.  Gradients land from
 * the last layer down, so a host optimizer can update layer L-1 while the backward
 * pass still works on the layers below.  SP_ERR_STATE for a layer that sends no
 * gradient (frozen, or no step yet).
 *
 * sp_weights_updated tells the handle that the caller has rewritten
 * layer_host_blobs[layer] (layer -1: every layer): a copy of it still in device
 * memory is forgotten and the next pass streams the layer in again.  Host order
 * only, no device work.  A layer's host blob may be rewritten (a) while none of the
 * handle's passes is in flight, or (b) during a training step once
 * sp_wait_gradient(layer) has returned: the step reads the layer for the last time
 * before it sends that gradient.  Skipping the call leaves stale weights in use for
 * as long as the layer stays resident. */
int sp_wait_gradient(sp_handle h, int layer);
int sp_weights_updated(sp_handle h, int layer);

/* Counters and (with SP_FLAG_TIMING) per-layer timings of the most recent call: how many bytes
 * crossed the link, how long each layer's copy and compute took and how much of the copy time lay
 * under compute -- the quantities the paper's evaluation reports per configuration (Sec. 4.2:
 * memory used and time per step for each k, k').  Synchronises the handle's streams when a timing
 * flag is on, otherwise returns at once. */
int sp_get_stats(sp_handle h, sp_stats* out);

/* Ends the streaming of this stack (Sec. 3.2.2: when execution is over the partitions' device
 * copies are given up; here the slots simply go back to the caller with the arena).  Waits for the
 * handle's streams, destroys its events, frees host bookkeeping.  Frees nothing the caller
 * allocated; the host weight blobs were never written.  Works on a FAILED handle. */
int sp_destroy(sp_handle h);

const char* sp_last_error(sp_handle h);

#ifdef __cplusplus
}
#endif
#endif /* SUPERPIPE_H */
