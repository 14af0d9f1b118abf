#!/usr/bin/env python3
"""Writes tests/golden/full_depth_<workload>.npz: the CPU oracle's output of a WHOLE workload
stack (every layer, full token count) on sampled token rows, plus per-layer norms.

    python tests/golden/make_full_depth_golden.py [--checkpoint DIR] [--legs plain,bf16] llama7b vith llama70b train1p3b

Two forward legs: "plain" (nothing rounded: the reference) and "bf16" (the oracle's optional mode
that rounds the contractions' operands to bf16; it measures, without any device code, how far
bf16 compute alone moves the output of the deep stack).  With --checkpoint a leg keeps its hidden
state and per-layer norms in DIR after every layer and a later run with the same DIR resumes
there (the 70B-shaped stack takes hours per leg); --legs runs a subset (the file is written once
the plain leg is complete; for a training workload `--legs bf16` adds the operand figures to a
stored result).

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
The bf16 leg adds: ops_y_rows [R, d] (its rows of y), ops_dev_all / ops_dev_rows (max |y_bf16 - y|
over all elements / over the sampled rows, as a fraction of y_absmax), ops_dev_fro (Frobenius
ratio), ops_rows_over_2e2 / ops_elems_over_2e2 (rows / elements whose deviation exceeds 2e-2 of
y_absmax).
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


class Leg:
    """One forward pass over the stack, resumable: hidden state and per-layer norms."""

    def __init__(self, name, tag, operands, x, dtype, ckpt_dir):
        self.tag, self.operands = tag, operands
        self.h, self.amax, self.fro = x.astype(dtype), [], []
        self.ckpt = os.path.join(ckpt_dir, f"{name}{'' if tag == 'plain' else '_' + tag}_state.npz") if ckpt_dir else None
        if self.ckpt and os.path.exists(self.ckpt):
            with np.load(self.ckpt) as c:
                self.h, self.amax, self.fro = c["h"].astype(dtype), list(c["amax"]), list(c["fro"])
            print(f"[{name}/{tag}] resumed after layer {len(self.amax)}", flush=True)

    @property
    def done(self):
        return len(self.amax)

    def step(self, wl, w, shape):
        self.h = O.layer_forward(self.h, wl, w.batch, w.seq, shape, operands=self.operands)
        self.amax.append(float(np.max(np.abs(self.h))))
        self.fro.append(float(np.sqrt(np.sum(self.h.astype(np.float64) ** 2))))
        if self.ckpt:
            np.savez(self.ckpt + ".tmp.npz", h=self.h, amax=np.array(self.amax), fro=np.array(self.fro))
            os.replace(self.ckpt + ".tmp.npz", self.ckpt)


def forward_legs(name, w, shape, x, distinct, dtype, ckpt_dir, tags):
    """Runs the requested forward legs layer by layer (weights of a layer are generated once for
    all legs that are at that layer).  Returns {tag: Leg}; a leg not requested is still loaded
    from its checkpoint if one exists, so that a later call can finish the job."""
    legs = {t: Leg(name, t, None if t == "plain" else t, x, dtype, ckpt_dir)
            for t in ("plain", "bf16") if t in tags or ckpt_dir}
    t0 = time.time()
    for l in range(w.n_layers):
        todo = [g for t, g in legs.items() if t in tags and g.done == l]
        if not todo:
            continue
        wl = {k: O.decode_bf16(v, dtype) for k, v in synth.make_layer(w, l % distinct).items()}
        for g in todo:
            g.step(wl, w, shape)
            print(f"[{name}/{g.tag}] layer {l + 1}/{w.n_layers}: max|h| {g.amax[-1]:.4g} ({time.time() - t0:.0f} s)", flush=True)
    return legs


def operand_stats(y, yb, rows):
    """How far rounding the contractions' operands to bf16 moves the oracle's own output."""
    d = np.abs(yb.astype(np.float64) - y.astype(np.float64))
    mx = float(np.max(np.abs(y)))
    return dict(ops_y_rows=yb[rows].astype(np.float32), ops_dev_all=float(d.max() / mx),
                ops_dev_rows=float(d[rows].max() / mx),
                ops_dev_fro=float(np.sqrt((d ** 2).sum() / (y.astype(np.float64) ** 2).sum())),
                ops_rows_over_2e2=int((d.max(axis=1) > 2e-2 * mx).sum()),
                ops_elems_over_2e2=int((d > 2e-2 * mx).sum()))


def run(name, dtype=np.float32, ckpt_dir=None, tags=("plain", "bf16")):
    w = synth.WORKLOADS[name]
    shape = oracle_shape(w)
    distinct = DISTINCT.get(name, w.n_layers)
    rows = sample_rows(w)
    x = synth.make_input(w).reshape(w.tokens, w.d_model)
    path = os.path.join(HERE, f"full_depth_{name}.npz")
    out = {"rows": rows, "distinct": distinct}
    t0 = time.time()
    if w.training and "plain" in tags:
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
        del grads, layers
        out.update(y_rows=y[rows].astype(np.float32), y_absmax=float(np.max(np.abs(y))),
                   y_fro=float(np.sqrt(np.sum(y.astype(np.float64) ** 2))),
                   dy_absmax=float(np.max(np.abs(y - x.astype(dtype)))),
                   layer_absmax=np.array([float(np.max(np.abs(y)))]),
                   layer_fro=np.array([float(np.sqrt(np.sum(y.astype(np.float64) ** 2)))]))
        if "bf16" in tags:
            # the operand-rounding leg is forward only (y, and through it the loss)
            legs = forward_legs(name, w, shape, x, distinct, dtype, ckpt_dir, ("bf16",))
            out.update(operand_stats(y, legs["bf16"].h, rows))
    elif w.training:
        # add the operand-rounding leg to a stored training result (its forward run twice here:
        # the plain output is needed whole for the all-element figures)
        with np.load(path) as old:
            out = {k: old[k] for k in old.files}
        legs = forward_legs(name, w, shape, x, distinct, dtype, ckpt_dir, ("plain", "bf16"))
        np.testing.assert_array_equal(legs["plain"].h[rows].astype(np.float32), out["y_rows"])
        out.update(operand_stats(legs["plain"].h, legs["bf16"].h, rows))
    else:
        legs = forward_legs(name, w, shape, x, distinct, dtype, ckpt_dir, tags)
        if "plain" not in legs or legs["plain"].done < w.n_layers:
            print(f"[{name}] the plain leg is not complete: nothing written; run again with it", flush=True)
            return
        g = legs["plain"]
        y = g.h
        out.update(y_rows=y[rows].astype(np.float32), y_absmax=float(np.max(np.abs(y))),
                   y_fro=float(np.sqrt(np.sum(y.astype(np.float64) ** 2))),
                   dy_absmax=float(np.max(np.abs(y - x.astype(dtype)))),
                   layer_absmax=np.array(g.amax), layer_fro=np.array(g.fro))
        if "bf16" in legs and legs["bf16"].done == w.n_layers:
            out.update(operand_stats(y, legs["bf16"].h, rows))
            print(f"[{name}] operands rounded to bf16 move the oracle's output by {out['ops_dev_all']:.3e} of its maximum "
                  f"({out['ops_dev_rows']:.3e} on the sampled rows, Frobenius {out['ops_dev_fro']:.3e})", flush=True)
    out["seconds"] = time.time() - t0
    np.savez(path, **out)
    print(f"[{name}] wrote {path} ({os.path.getsize(path)} bytes, {time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    argv = sys.argv[1:]
    ckpt_dir, tags = None, ("plain", "bf16")
    while argv and argv[0].startswith("--"):
        if argv[0] == "--checkpoint":
            ckpt_dir = argv[1]
            os.makedirs(ckpt_dir, exist_ok=True)
        elif argv[0] == "--legs":
            tags = tuple(argv[1].split(","))
        else:
            raise SystemExit(f"unknown option {argv[0]}")
        argv = argv[2:]
    for n in argv or ["llama7b", "vith", "train1p3b", "llama70b"]:
        run(n, ckpt_dir=ckpt_dir, tags=tags)
