"""ctypes binding of libsuperpipe.so -- argument marshalling only.

Same names as include/superpipe.h and include/superpipe_kernels.h.  torch is
used here for device memory, pinned host memory and streams, nothing else:
every step of the path runs in the library's kernels.  There is no fallback:
if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# torch first: its wheel bundles a HIP runtime, and the library must bind to the
# SAME runtime instance that allocates the pinned and device memory it is handed.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsuperpipe.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first with `python -m paper_2410_08791_amd.build` "
        "(there is no CPU fallback for the HIP path)")
lib = C.CDLL(LIB_PATH)

SP_OK, SP_ERR_INVALID_ARG, SP_ERR_BUDGET, SP_ERR_NOT_PINNED, SP_ERR_HIP, SP_ERR_STATE, SP_ERR_SHAPE = 0, -1, -2, -3, -4, -5, -6
SP_DECODER_SWIGLU_RMS, SP_ENCODER_GELU_LN = 0, 1
SP_FLAG_TRAINING, SP_FLAG_TIMING, SP_FLAG_POISON, SP_FLAG_NO_OVERLAP, SP_FLAG_WRAP_PREFETCH = 1, 2, 4, 8, 16
SP_FLAG_KERNEL_TIMING = 32
SP_FLAG_KEEP_ACTIVATIONS = 64
SP_FLAG_DELAY = 128
SP_FLAG_OP_TIMING = 256
SP_OP_NAMES = ["norm", "gemm_qkv", "attention", "gemm_o", "gemm_ffn1", "act", "gemm_ffn2", "loss", "gemm_dw", "gemm_dx",
               "act_bwd", "norm_bwd", "attention_bwd", "bias_grad", "copy"]
SP_PIN_AUTO = -1
SP_MAX_TRACE_LAYERS = 256
EPI_BF16, EPI_RESID_F32, EPI_GELU_BF16, EPI_SWIGLU_BF16, EPI_F32 = 0, 1, 2, 3, 4

TENSOR_NAMES = {
    SP_DECODER_SWIGLU_RMS: ["g1", "wqkv", "wo", "g2", "wgu", "wd"],
    SP_ENCODER_GELU_LN: ["ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"],
}


class sp_stack_desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_int32), ("d_model", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("arch", C.c_int32), ("causal", C.c_int32),
                ("norm_eps", C.c_float), ("max_batch", C.c_int32), ("max_seq", C.c_int32)]


class sp_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("resident_window_k", C.c_int32), ("prefetch_depth_p", C.c_int32),
                ("gpu_budget_bytes", C.c_uint64), ("device_arena", C.c_void_p), ("compute_stream", C.c_void_p),
                ("h2d_stream", C.c_void_p), ("d2h_stream", C.c_void_p), ("flags", C.c_uint32),
                ("frozen_layers", C.c_int32), ("pinned_layers", C.c_int32), ("units_per_layer", C.c_int32),
                ("delay_us", C.c_int32)]


class sp_plan(C.Structure):
    _fields_ = [("n_slots", C.c_int32), ("k_eff", C.c_int32), ("p_eff", C.c_int32), ("fully_resident", C.c_int32),
                ("slot_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64), ("arena_bytes_used", C.c_uint64),
                ("n_pinned", C.c_int32), ("units_per_layer", C.c_int32), ("pinned_bytes", C.c_uint64)]


_F = C.c_float * SP_MAX_TRACE_LAYERS


class sp_stats(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("plan", sp_plan), ("calls", C.c_uint64),
                ("h2d_copies", C.c_uint64), ("h2d_bytes", C.c_uint64), ("d2h_copies", C.c_uint64),
                ("d2h_bytes", C.c_uint64), ("last_h2d_copies", C.c_uint64), ("last_h2d_bytes", C.c_uint64),
                ("n_timed", C.c_int32), ("copy_begin_ms", _F), ("copy_end_ms", _F), ("comp_begin_ms", _F),
                ("comp_end_ms", _F), ("copy_busy_ms", C.c_float), ("copy_hidden_ms", C.c_float),
                ("compute_busy_ms", C.c_float), ("wall_ms", C.c_float),
                ("big_gemm_launches", C.c_uint32), ("big_gemm_ms_sum", C.c_float),
                ("big_gemm_m", C.c_int32), ("big_gemm_n", C.c_int32), ("big_gemm_k", C.c_int32),
                ("op_ms", C.c_float * 16), ("op_launches", C.c_uint32 * 16), ("n_ops", C.c_int32)]


class sp_sched_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layer", C.c_int32), ("slot", C.c_int32), ("wait_layer", C.c_int32),
                ("pass_", C.c_int32)]


class sp_layer_cost(C.Structure):
    _fields_ = [("copy_ms", C.c_double), ("fwd_ms", C.c_double), ("bwd_ms", C.c_double), ("grad_ms", C.c_double)]


_P = C.POINTER
_sig = {
    "sp_simulate_call_ms": (C.c_double, [C.c_int] * 7 + [_P(sp_layer_cost)]),
    "sp_autotune": (C.c_int, [_P(sp_stack_desc), C.c_uint64, C.c_int, C.c_int, _P(sp_layer_cost), C.c_double,
                              _P(C.c_int), _P(C.c_int), _P(C.c_int), _P(C.c_double)]),
    "sp_autotune_units": (C.c_int, [_P(sp_stack_desc), C.c_uint64, C.c_int, C.c_int, _P(sp_layer_cost), C.c_double,
                                    _P(C.c_int), _P(C.c_int), _P(C.c_int), _P(C.c_int), _P(C.c_double)]),
    "sp_num_tensors": (C.c_int, [_P(sp_stack_desc)]),
    "sp_tensor_offset": (C.c_size_t, [_P(sp_stack_desc), C.c_int]),
    "sp_tensor_elems": (C.c_size_t, [_P(sp_stack_desc), C.c_int]),
    "sp_layer_blob_bytes": (C.c_size_t, [_P(sp_stack_desc)]),
    "sp_layer_grad_bytes": (C.c_size_t, [_P(sp_stack_desc)]),
    "sp_workspace_bytes": (C.c_size_t, [_P(sp_stack_desc), C.c_int]),
    "sp_make_plan": (C.c_int, [_P(sp_stack_desc), C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int, _P(sp_plan)]),
    "sp_make_plan_units": (C.c_int, [_P(sp_stack_desc), C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int,
                                     _P(sp_plan)]),
    "sp_unit_range": (C.c_int, [_P(sp_stack_desc), C.c_int, C.c_int, _P(C.c_uint64), _P(C.c_uint64)]),
    "sp_trace_schedule": (C.c_int, [C.c_int] * 7 + [_P(sp_sched_op), C.c_int]),
    "sp_trace_schedule_updated": (C.c_int, [C.c_int] * 7 + [_P(C.c_int), C.c_int, _P(sp_sched_op), C.c_int]),
    "sp_create": (C.c_int, [_P(C.c_void_p), _P(sp_stack_desc), _P(C.c_void_p), _P(sp_config)]),
    "sp_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]),
    "sp_kv_cache_bytes": (C.c_size_t, [_P(sp_stack_desc), C.c_int, C.c_int]),
    "sp_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "sp_decode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "spk_kv_append": (C.c_int, [C.c_void_p] * 4 + [C.c_int] * 7),
    "spk_decode_attention": (C.c_int, [C.c_void_p] * 5 + [C.c_int] * 6),
    "spk_layernorm_bwd": (C.c_int, [C.c_void_p] * 9 + [C.c_int, C.c_int, C.c_float]),
    "spk_gelu": (C.c_int, [C.c_void_p] * 3 + [C.c_size_t]),
    "spk_gelu_bwd": (C.c_int, [C.c_void_p] * 3 + [C.c_size_t]),
    "spk_colsum_bf16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "sp_forward_backward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      _P(C.c_void_p), C.c_int, C.c_int]),
    "sp_wait_gradient": (C.c_int, [C.c_void_p, C.c_int]),
    "sp_weights_updated": (C.c_int, [C.c_void_p, C.c_int]),
    "sp_get_stats": (C.c_int, [C.c_void_p, _P(sp_stats)]),
    "sp_destroy": (C.c_int, [C.c_void_p]),
    "sp_last_error": (C.c_char_p, [C.c_void_p]),
    "spk_norm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float]),
    "spk_gemm": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                           C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]),
    "spk_gemm_plan": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]),
    "spk_swiglu": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]),
    "spk_attention": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                C.c_int, C.c_int, C.c_int, C.c_int]),
    "spk_mse": (C.c_int, [C.c_void_p] * 7 + [C.c_size_t]),
    "spk_swiglu_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]),
    "spk_rmsnorm_bwd": (C.c_int, [C.c_void_p] * 8 + [C.c_int, C.c_int, C.c_float]),
    "spk_rmsnorm_bwd_static": (C.c_int, [C.c_void_p] * 7 + [C.c_int, C.c_int, C.c_float]),
    "spk_rmsnorm_bwd_static_max_d": (C.c_int, []),
    "spk_attention_bwd_scratch_bytes": (C.c_size_t, [C.c_int] * 5),
    "spk_attention_bwd": (C.c_int, [C.c_void_p] * 7 + [C.c_int] * 6),
}
for _n, (_r, _a) in _sig.items():
    _f = getattr(lib, _n)          # AttributeError here = header/library mismatch
    _f.restype, _f.argtypes = _r, _a
    globals()[_n] = _f
EXPORTS = sorted(_sig)


class SuperpipeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sp_status {code}: {msg}")
        self.code = code


def make_desc(w, max_batch=None, max_seq=None, n_layers=None):
    """sp_stack_desc from a synth.Workload-like object."""
    arch = SP_DECODER_SWIGLU_RMS if w.arch == "decoder" else SP_ENCODER_GELU_LN
    return sp_stack_desc(C.sizeof(sp_stack_desc), w.n_layers if n_layers is None else n_layers, w.d_model,
                         w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn, arch, int(w.causal), w.norm_eps,
                         w.batch if max_batch is None else max_batch, w.seq if max_seq is None else max_seq)


def blob_views(desc, blob_u8: np.ndarray):
    """{tensor name: uint16 view} into one layer blob (a uint8 numpy array)."""
    names = TENSOR_NAMES[desc.arch]
    out = {}
    for i, n in enumerate(names):
        off = sp_tensor_offset(C.byref(desc), i)
        cnt = sp_tensor_elems(C.byref(desc), i)
        out[n] = blob_u8[off:off + 2 * cnt].view(np.uint16)
    return out


def grad_views(desc, gblob_u8: np.ndarray):
    """{tensor name: float32 view} into one layer's fp32 gradient blob."""
    names = TENSOR_NAMES[desc.arch]
    out = {}
    for i, n in enumerate(names):
        off = 2 * sp_tensor_offset(C.byref(desc), i)
        cnt = sp_tensor_elems(C.byref(desc), i)
        out[n] = gblob_u8[off:off + 4 * cnt].view(np.float32)
    return out


def plan(desc, k, p, budget, training=False, pinned=0):
    pl = sp_plan()
    rc = sp_make_plan(C.byref(desc), k, p, pinned, budget, int(training), C.byref(pl))
    return rc, pl


def trace_schedule(n_layers, n_slots, p_eff, training=False, wrap=False, passes=1, pinned=0, frozen=0,
                   updated=()):
    """updated: layers whose host weights the caller rewrites between calls."""
    training = int(bool(training)) + (frozen if training else 0)
    upd = (C.c_int * max(1, len(updated)))(*updated)
    args = (n_layers, n_slots, pinned, p_eff, int(training), int(wrap), passes, upd, len(updated))
    n = sp_trace_schedule_updated(*args, None, 0)
    if n < 0:
        raise SuperpipeError(n, "sp_trace_schedule")
    ops = (sp_sched_op * n)()
    sp_trace_schedule_updated(*args, ops, n)
    return [(o.kind, o.layer, o.slot, o.wait_layer, o.pass_) for o in ops]


def simulate_call_ms(n_layers, n_slots, p_eff, cost, training=False, wrap=False, calls=3, pinned=0):
    """Modelled duration of the last of `calls` calls; cost = (copy, fwd, bwd, grad) in ms."""
    c = sp_layer_cost(*cost)
    return sp_simulate_call_ms(n_layers, n_slots, pinned, p_eff, int(training), int(wrap), calls, C.byref(c))


def autotune(desc, budget_bytes, cost, training=0, wrap=False, tolerance=0.02):
    """(k, p, pinned layers, modelled ms) for the smallest window within `tolerance` of the best
    modelled time."""
    c = sp_layer_cost(*cost)
    k, p, r, ms = C.c_int(), C.c_int(), C.c_int(), C.c_double()
    rc = sp_autotune(C.byref(desc), budget_bytes, int(training), int(wrap), C.byref(c), tolerance,
                     C.byref(k), C.byref(p), C.byref(r), C.byref(ms))
    if rc != SP_OK:
        raise SuperpipeError(rc, "sp_autotune")
    return k.value, p.value, r.value, ms.value


def autotune_units(desc, budget_bytes, cost, training=0, wrap=False, tolerance=0.02):
    """(units per layer, k, p, pinned units, modelled ms): sp_autotune's choice against a layer
    streamed as three units."""
    c = sp_layer_cost(*cost)
    u, k, p, r, ms = C.c_int(), C.c_int(), C.c_int(), C.c_int(), C.c_double()
    rc = sp_autotune_units(C.byref(desc), budget_bytes, int(training), int(wrap), C.byref(c), tolerance,
                           C.byref(u), C.byref(k), C.byref(p), C.byref(r), C.byref(ms))
    if rc != SP_OK:
        raise SuperpipeError(rc, "sp_autotune_units")
    return u.value, k.value, p.value, r.value, ms.value


def layer_costs(st, n_layers, training=False, grad_ms=0.0):
    """(copy, fwd, bwd, grad) per-layer medians in ms from a SP_FLAG_TIMING sp_stats."""
    n = st.n_timed
    comp = [st.comp_end_ms[j] - st.comp_begin_ms[j] for j in range(n)]
    copy = [st.copy_end_ms[j] - st.copy_begin_ms[j] for j in range(n) if st.copy_begin_ms[j] >= 0]
    med = lambda v: float(np.median(v)) if len(v) else 0.0
    fwd = comp[:n_layers] if training else comp
    bwd = comp[n_layers:2 * n_layers] if training else []
    return med(copy), med(fwd), med(bwd), float(grad_ms)


def pinned_blobs(w, desc, n_layers=None, pool=None):
    """Seeded weights straight into pinned host blobs.  Returns (torch tensors, per-layer views)."""
    import torch
    from . import synth
    nbytes = sp_layer_blob_bytes(C.byref(desc))
    L = desc.n_layers if n_layers is None else n_layers
    blobs, views = [], []
    for l in range(L):
        t = torch.zeros(nbytes, dtype=torch.uint8, pin_memory=True)
        v = blob_views(desc, t.numpy())
        v = {n: v[n].reshape(shape) for n, shape, _ in synth.tensor_specs(w)}
        synth.fill_layer(v, w, l, pool=pool)
        blobs.append(t)
        views.append(v)
    return blobs, views


_STREAMS = {}


def _device_streams(torch, device):
    """One (compute, h2d, d2h) stream trio per device, shared by every Engine of the
    process.  HIP multiplexes a process's streams onto a few hardware queues (4 by
    default); once there are more streams than queues a copy stream lands on the queue
    of another stream and its copies serialise behind that stream's kernels (measured:
    +23 % on the training step).  Three streams plus the default one stay within that."""
    key = (device.type, device.index if device.index is not None else torch.cuda.current_device())
    if key not in _STREAMS:
        _STREAMS[key] = tuple(torch.cuda.Stream(device=device) for _ in range(3))
    return _STREAMS[key]


class Engine:
    """Owns an sp_handle plus the torch-allocated arena and streams it runs on."""

    def __init__(self, desc, blobs, k, p, budget_bytes=None, budget_layers=None, flags=0, device="cuda:0",
                 pinned=0, frozen=0, units=1, delay_us=0):
        import torch
        self.torch = torch
        self.desc = desc
        self.blobs = blobs                      # keep the pinned tensors alive
        training = bool(flags & SP_FLAG_TRAINING)
        ws = sp_workspace_bytes(C.byref(desc), (2 if flags & SP_FLAG_KEEP_ACTIVATIONS else 1) if training else 0)
        slot = (sp_layer_blob_bytes(C.byref(desc)) + 4095) // 4096 * 4096
        if budget_bytes is None:
            nl = budget_layers if budget_layers else min(k + p + max(pinned, 0), desc.n_layers)
            budget_bytes = ws + nl * slot
        self.budget_bytes = int(budget_bytes)
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            # torch hands out 512-byte aligned blocks; take 4 KiB of slack and align by hand
            self._arena_raw = torch.empty(self.budget_bytes + 4096, dtype=torch.uint8, device=self.device)
            skew = (-self._arena_raw.data_ptr()) % 4096
            self.arena = self._arena_raw[skew:skew + self.budget_bytes]
            self.compute, self.h2d, d2h = _device_streams(torch, self.device)
            self.d2h = d2h if training else None
        assert self.arena.data_ptr() % 4096 == 0
        ptrs = (C.c_void_p * len(blobs))(*[b.data_ptr() for b in blobs])
        cfg = sp_config(C.sizeof(sp_config), k, p, self.budget_bytes, self.arena.data_ptr(),
                        self.compute.cuda_stream, self.h2d.cuda_stream,
                        self.d2h.cuda_stream if training else None, flags, frozen, pinned, units, delay_us)
        self.handle = C.c_void_p()
        rc = sp_create(C.byref(self.handle), C.byref(desc), ptrs, C.byref(cfg))
        if rc != SP_OK:
            raise SuperpipeError(rc, sp_last_error(None).decode())

    def _check(self, rc):
        if rc != SP_OK:
            raise SuperpipeError(rc, sp_last_error(self.handle).decode())

    def forward(self, x, y, B, S):
        """x, y: fp32 cuda tensors [B,S,d]; enqueues on self.compute (after whatever
        torch's current stream has enqueued so far, e.g. the producer of x)."""
        self.compute.wait_stream(self.torch.cuda.current_stream(self.device))
        self._check(sp_forward(self.handle, x.data_ptr(), y.data_ptr(), B, S))

    def prefill(self, x, y, kv_cache, B, S, max_len):
        """x, y: fp32 cuda [B,S,d]; kv_cache: cuda uint8 tensor of sp_kv_cache_bytes."""
        self.compute.wait_stream(self.torch.cuda.current_stream(self.device))
        self._check(sp_prefill(self.handle, x.data_ptr(), y.data_ptr(), kv_cache.data_ptr(), B, S, max_len))

    def decode(self, x, y, kv_cache, B, pos, max_len):
        """x, y: fp32 cuda [B,d]: one new token per sequence at position pos."""
        self.compute.wait_stream(self.torch.cuda.current_stream(self.device))
        self._check(sp_decode(self.handle, x.data_ptr(), y.data_ptr(), kv_cache.data_ptr(), B, pos, max_len))

    def forward_backward(self, x, target, y, loss, dx, grad_blobs, B, S):
        ptrs = (C.c_void_p * len(grad_blobs))(*[g.data_ptr() for g in grad_blobs])
        self.compute.wait_stream(self.torch.cuda.current_stream(self.device))
        self._check(sp_forward_backward(self.handle, x.data_ptr(), target.data_ptr(),
                                        y.data_ptr() if y is not None else None, loss.data_ptr(),
                                        dx.data_ptr() if dx is not None else None, ptrs, B, S))

    def wait_gradient(self, layer):
        self._check(sp_wait_gradient(self.handle, layer))

    def weights_updated(self, layer=-1):
        self._check(sp_weights_updated(self.handle, layer))

    def sync(self):
        self.compute.synchronize()
        self.h2d.synchronize()
        if self.d2h is not None:
            self.d2h.synchronize()

    def stats(self):
        st = sp_stats()
        self._check(sp_get_stats(self.handle, C.byref(st)))
        return st

    def destroy(self):
        if self.handle:
            rc = sp_destroy(self.handle)
            self.handle = C.c_void_p()
            return rc
        return SP_ERR_STATE

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
