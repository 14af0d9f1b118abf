#!/usr/bin/env python3
"""Writes tests/golden/full_depth_<workload>.npz: the CPU oracle's output of a WHOLE workload
stack (every layer, full token count) on sampled token rows, plus per-layer norms.

    python tests/golden/make_full_depth_golden.py [--checkpoint DIR] llama7b vith llama70b train1p3b

With --checkpoint an inference run keeps its hidden state and per-layer norms in DIR after every
layer and a later run with the same DIR resumes there (the 70B-shaped stack takes hours).

This script calls only oracle/ and the seeded input generator (synth.py); nothing in the files it
writes comes from the HIP path.  The full-depth runs take minutes to hours of CPU time (the 80-layer
70B-shaped stack is ~7 TFLOP per layer), which is why their results are stored instead of being
recomputed inside the GPU tests: the GPU test runs the same seeded workload through the library
and compares the sampled rows, to the same max-relative-error bound as the small cases.

Stored per workload (float32 oracle arithmetic on the exact bf16 weight values, no rounding of
any intermediate):
    rows        int64 [R]        sampled token rows (first, last, the ragged tail, seeded others)
    y_rows      float32 [R, d]   rows of y = h_L
    y_absmax    float            max |y| over ALL tokens (the error norm's denominator)
    y_fro       float            Frobenius norm of y
    dy_absmax   float            max |y - x| over all tokens (what the stack itself contributed)
    layer_absmax, layer_fro      float64 [L]  the same two norms of every h_{l+1}
    distinct    int              layer l uses the seeded weights of layer l % distinct
Training workloads add: loss, dx_rows [R, d], dx_absmax, and per layer and weight tensor the
gradient's absmax and Frobenius norm and 64 sampled entries (flat indices seeded per tensor).
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import stack_oracle as O  # noqa: E402
from paper_2410_08791_amd import synth  # noqa: E402

N_ROWS = 16
N_GRAD_SAMPLES = 64
# host RAM: the 70B-shaped stack cycles 16 distinct layers, as the benchmark does
DISTINCT = {"llama70b": 16}


def sample_rows(w):
    T = w.tokens
    fixed = {0, 1, T - 1, T - 2, T // 2, (T // 256) * 256 % T, max(T - 63, 0)}
    rng = np.random.default_rng(20241008)
    while len(fixed) < min(N_ROWS, T):
        fixed.add(int(rng.integers(0, T)))
    return np.array(sorted(fixed), dtype=np.int64)


def grad_sample_index(size, layer, tidx):
    rng = np.random.default_rng([20241008, layer, tidx])
    return rng.integers(0, size, size=min(N_GRAD_SAMPLES, size)).astype(np.int64)


def oracle_shape(w):
    return O.StackShape(w.arch, w.n_layers, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn,
                        w.causal, w.norm_eps)


def run(name, dtype=np.float32, ckpt_dir=None):
    w = synth.WORKLOADS[name]
    shape = oracle_shape(w)
    distinct = DISTINCT.get(name, w.n_layers)
    rows = sample_rows(w)
    x = synth.make_input(w).reshape(w.tokens, w.d_model)
    out = {"rows": rows, "distinct": distinct}
    t0 = time.time()
    if not w.training:
        h = x.astype(dtype)
        amax, fro = [], []
        ckpt = os.path.join(ckpt_dir, f"{name}_state.npz") if ckpt_dir else None
        if ckpt and os.path.exists(ckpt):
            with np.load(ckpt) as c:
                h, amax, fro = c["h"].astype(dtype), list(c["amax"]), list(c["fro"])
            print(f"[{name}] resumed after layer {len(amax)}", flush=True)
        for l in range(len(amax), w.n_layers):
            wl = {k: O.decode_bf16(v, dtype) for k, v in synth.make_layer(w, l % distinct).items()}
            h = O.layer_forward(h, wl, w.batch, w.seq, shape)
            amax.append(float(np.max(np.abs(h))))
            fro.append(float(np.sqrt(np.sum(h.astype(np.float64) ** 2))))
            print(f"[{name}] layer {l + 1}/{w.n_layers}: max|h| {amax[-1]:.4g} ({time.time() - t0:.0f} s)", flush=True)
            if ckpt:
                np.savez(ckpt + ".tmp.npz", h=h, amax=np.array(amax), fro=np.array(fro))
                os.replace(ckpt + ".tmp.npz", ckpt)
        y = h
    else:
        t = synth.make_input(w, "target")
        layers = [synth.make_layer(w, l % distinct) for l in range(w.n_layers)]
        y, loss, dx, grads = O.stack_forward_backward(x, t, layers, w.batch, w.seq, shape, dtype=dtype)
        out["loss"] = float(loss)
        out["dx_rows"] = dx[rows].astype(np.float32)
        out["dx_absmax"] = float(np.max(np.abs(dx)))
        names = [n for n, _, _ in synth.tensor_specs(w)]
        g_absmax = np.zeros((w.n_layers, len(names)))
        g_fro = np.zeros((w.n_layers, len(names)))
        g_samples = np.zeros((w.n_layers, len(names), N_GRAD_SAMPLES), dtype=np.float32)
        for l in range(w.n_layers):
            for ti, n in enumerate(names):
                g = np.asarray(grads[l][n]).reshape(-1)
                g_absmax[l, ti] = np.max(np.abs(g))
                g_fro[l, ti] = np.sqrt(np.sum(g.astype(np.float64) ** 2))
                idx = grad_sample_index(g.size, l, ti)
                g_samples[l, ti, :idx.size] = g[idx]
        out.update(grad_absmax=g_absmax, grad_fro=g_fro, grad_samples=g_samples)
        amax, fro = [float(np.max(np.abs(y)))], [float(np.sqrt(np.sum(y.astype(np.float64) ** 2)))]
    out.update(y_rows=y[rows].astype(np.float32), y_absmax=float(np.max(np.abs(y))),
               y_fro=float(np.sqrt(np.sum(y.astype(np.float64) ** 2))),
               dy_absmax=float(np.max(np.abs(y - x.astype(dtype)))),
               layer_absmax=np.array(amax), layer_fro=np.array(fro), seconds=time.time() - t0)
    path = os.path.join(HERE, f"full_depth_{name}.npz")
    np.savez(path, **out)
    print(f"[{name}] wrote {path} ({os.path.getsize(path)} bytes, {time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    argv = sys.argv[1:]
    ckpt_dir = None
    if argv[:1] == ["--checkpoint"]:
        ckpt_dir = argv[1]
        os.makedirs(ckpt_dir, exist_ok=True)
        argv = argv[2:]
    for n in argv or ["llama7b", "vith", "train1p3b", "llama70b"]:
        run(n, ckpt_dir=ckpt_dir)
