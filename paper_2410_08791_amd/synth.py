"""Seeded synthetic workloads: shapes, weight tensors and inputs.

This module only *generates data*.  It holds none of the method's arithmetic
and is the one module that both the test oracle's callers and the HIP path's
callers may use, so that both see the same bytes.

The paper evaluates on trained LLaMA-2 / ViT-bigG / Stable Diffusion
checkpoints (Sec. 4.1); none of those exist here, so seeded Gaussian stacks of
the same families and shapes stand in for them: bf16 weight matrices with
standard deviation 0.02, norm gains 1 + N(0, 0.02), biases N(0, 0.02), fp32
inputs N(0, 1).  Every tensor is drawn from its own Philox stream keyed by
(seed, layer, tensor index), rounded once to bfloat16 (round to nearest even);
both consumers read those same 16-bit patterns.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

DECODER = "decoder"
ENCODER = "encoder"

_CHUNK = 1 << 22  # elements drawn per Philox stream segment


@dataclass(frozen=True)
class Workload:
    name: str
    arch: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    causal: bool
    batch: int
    seq: int
    k: int = 1                 # resident window
    p: int = 1                 # prefetch depth
    budget_layers: int = 0     # HBM weight budget in layer slots (0 = k + p)
    training: bool = False
    gen: int = 0               # > 0: decode workload, `seq` prompt positions then this many new tokens
    norm_eps: float = 1e-5
    seed: int = 0

    @property
    def tokens(self):
        return self.batch * self.seq

    def with_(self, **kw):
        return replace(self, **kw)


WORKLOADS = {
    # 4 pre-RMSNorm decoder layers, the case the oracle finishes in milliseconds
    "tiny": Workload("tiny", DECODER, 4, 256, 4, 4, 64, 1024, True, 2, 128, k=1, p=1),
    # LLaMA-2-7B shape: 32 repeated layers (Sec. 3.2.1 names this split)
    "llama7b": Workload("llama7b", DECODER, 32, 4096, 32, 32, 128, 11008, True, 1, 2048,
                        k=2, p=2, budget_layers=4),
    # ViT-H shape, stands in for the paper's ViT-bigG rows
    "vith": Workload("vith", ENCODER, 32, 1280, 16, 16, 80, 5120, False, 64, 257, k=2, p=1),
    # LLaMA-70B shape with grouped-query heads
    "llama70b": Workload("llama70b", DECODER, 80, 8192, 64, 8, 128, 28672, True, 4, 1024,
                         k=2, p=2),
    # the same stack generating tokens: 8 sequences, 512-position prompt, one token per step
    "llama7b_decode": Workload("llama7b_decode", DECODER, 32, 4096, 32, 32, 128, 11008, True, 8, 512,
                               k=2, p=2, budget_layers=4, gen=32),
    # 1.3B-shaped training step
    "train1p3b": Workload("train1p3b", DECODER, 24, 2048, 16, 16, 128, 5504, True, 8, 1024,
                          k=2, p=1, training=True),
    # ViT-H-shaped training step (the paper's ViT rows of Table 2), 32 images per step
    "trainvith": Workload("trainvith", ENCODER, 32, 1280, 16, 16, 80, 5120, False, 32, 257,
                          k=2, p=1, training=True),
}


def tensor_specs(w: Workload):
    """[(name, shape, kind)] in the fixed per-layer order; kind in matrix|gain|bias."""
    d, f = w.d_model, w.d_ffn
    nq = w.n_q_heads * w.head_dim
    nkv = w.n_kv_heads * w.head_dim
    if w.arch == DECODER:
        return [("g1", (d,), "gain"),
                ("wqkv", (nq + 2 * nkv, d), "matrix"),
                ("wo", (d, nq), "matrix"),
                ("g2", (d,), "gain"),
                ("wgu", (2 * f, d), "matrix"),
                ("wd", (d, f), "matrix")]
    return [("ln1_g", (d,), "gain"), ("ln1_b", (d,), "bias"),
            ("wqkv", (nq + 2 * nkv, d), "matrix"), ("bqkv", (nq + 2 * nkv,), "bias"),
            ("wo", (d, nq), "matrix"), ("bo", (d,), "bias"),
            ("ln2_g", (d,), "gain"), ("ln2_b", (d,), "bias"),
            ("w1", (f, d), "matrix"), ("b1", (f,), "bias"),
            ("w2", (d, f), "matrix"), ("b2", (d,), "bias")]


def params_per_layer(w: Workload):
    return sum(int(np.prod(s)) for _, s, _ in tensor_specs(w))


def f32_to_bf16_bits(a):
    """float32 -> bfloat16 bit patterns, round to nearest even (inputs are finite)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _fill_chunk(out_flat, seed, layer, tidx, chunk, kind):
    lo = chunk * _CHUNK
    hi = min(out_flat.size, lo + _CHUNK)
    rng = np.random.Generator(np.random.Philox(key=[(seed << 32) | (layer << 8) | tidx, chunk]))
    v = rng.standard_normal(hi - lo, dtype=np.float32)
    v *= np.float32(0.02)
    if kind == "gain":
        v += np.float32(1.0)
    out_flat[lo:hi] = f32_to_bf16_bits(v)


def fill_layer(views, w: Workload, layer: int, seed=None, pool=None):
    """Fill {name: uint16 array} (e.g. views into a pinned blob) for one layer."""
    seed = w.seed if seed is None else seed
    jobs = []
    for tidx, (name, shape, kind) in enumerate(tensor_specs(w)):
        flat = views[name].reshape(-1)
        assert flat.size == int(np.prod(shape)) and flat.dtype == np.uint16, name
        for c in range((flat.size + _CHUNK - 1) // _CHUNK):
            jobs.append((flat, seed, layer, tidx, c, kind))
    if pool is None:
        for j in jobs:
            _fill_chunk(*j)
    else:
        list(pool.map(lambda j: _fill_chunk(*j), jobs))


def make_layer(w: Workload, layer: int, seed=None):
    """Allocate and fill one layer's tensors: {name: uint16 bf16 bits}."""
    views = {n: np.empty(s, dtype=np.uint16) for n, s, _ in tensor_specs(w)}
    fill_layer(views, w, layer, seed)
    return views


def make_layers(w: Workload, seed=None, n_layers=None):
    return [make_layer(w, l, seed) for l in range(w.n_layers if n_layers is None else n_layers)]


def make_pool(threads=8):
    return ThreadPoolExecutor(max_workers=threads)


def make_input(w: Workload, what="x", seed=None):
    """fp32 N(0,1) tensor [B, S, d]; `what` ('x' or 'target') selects the stream."""
    seed = w.seed if seed is None else seed
    sid = {"x": 1, "target": 2}[what]
    rng = np.random.Generator(np.random.Philox(key=[(seed << 32) | 0xFFFF00 | sid, 0]))
    return rng.standard_normal((w.batch, w.seq, w.d_model), dtype=np.float32)
