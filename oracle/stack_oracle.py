"""Plain CPU oracle for the layer stack that Superpipeline streams.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg call it.
It shares no code with the HIP library: no layouts, tables, helpers or
constants are common to the two, and neither imports the other.

What it computes.  The paper's method (Sec. 3.2-3.3) moves layers between host
and device but leaves the model's arithmetic untouched: its result is that of
the un-offloaded model (Sec. 4.2, Sec. 4.2.2 and Sec. 6 all state that outputs
equal those of the standard mode).  The oracle is therefore the plain definition of the
layer stack, with every weight "resident": no window, no slots, no streams.
A partition is one repeated transformer layer (Sec. 3.2.1); training repeats
the process for the backward pass (Sec. 3.3), here the analytic gradient of a
mean-squared-error loss.

Two layer kinds, fixed by the build's workload list (the paper names the model
families, Sec. 4.1, but prints no layer equations -- the definitions below are
the standard ones for those families; parity of these definitions against the
paper itself is therefore "parity unpinned"; they are pinned against
brute-force scalar definitions, closed forms and finite differences instead):

  decoder (pre-RMSNorm, SwiGLU, optional causal mask, grouped-query heads)
      a  = rmsnorm(h, g1)            q,k,v = split(a Wqkv^T)
      h  = h + attn(q,k,v) Wo^T
      m  = rmsnorm(h, g2)            g,u = split(m Wgu^T)
      h  = h + (silu(g) * u) Wd^T
  encoder (pre-LayerNorm, biased linears, exact-erf GELU, no mask)
      a  = layernorm(h, ln1_g, ln1_b)   q,k,v = split(a Wqkv^T + bqkv)
      h  = h + attn(q,k,v) Wo^T + bo
      m  = layernorm(h, ln2_g, ln2_b)
      h  = h + gelu(m W1^T + b1) W2^T + b2

Weights are given per layer as a dict name -> array.  Matrices are [out, in]
(y = x W^T).  Wqkv stacks query rows, then key rows, then value rows; Wgu
stacks gate rows, then up rows.  Arrays of dtype uint16 are taken as bfloat16
bit patterns and widened exactly.  No intermediate is ever rounded to bf16:
arithmetic is carried out in `dtype` (float32 as the benchmark spec of the
oracle says; float64 for the pins and small parity cases).

One optional departure, off by default: `operands="bf16"` rounds the operands
of the dense contractions (normed activations, q/k/v, attention weights,
attention output, SwiGLU/GELU output) to bfloat16, round-to-nearest-even,
where a bf16 matrix pipeline has to; accumulation stays in `dtype`.  It answers
one question without any device code: how far does "bf16 compute, fp32
accumulate" alone move the output of a deep stack away from the exact result?
The plain mode remains the reference every parity test compares against.

Library primitives used as steps: numpy matmul, exp, sqrt, tanh-free erf
(scipy.special.erf).  No blocking, fusion or reordering.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
from scipy.special import erf as _erf

DECODER = "decoder"
ENCODER = "encoder"


@dataclass(frozen=True)
class StackShape:
    arch: str          # DECODER or ENCODER
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    causal: bool
    norm_eps: float = 1e-5


def decode_bf16(a, dtype):
    """Widen bfloat16 bit patterns (uint16) exactly; pass floats through."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype)
    return a.astype(dtype, copy=False)


def round_bf16(x):
    """Nearest bfloat16 (ties to even) of every element, returned in x's dtype.  Finite inputs."""
    x = np.asarray(x)
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(x.dtype, copy=False)


def _operand(x, operands):
    if operands is None:
        return x
    if operands == "bf16":
        return round_bf16(x)
    raise ValueError(operands)


def _weights(layer, dtype):
    return {k: decode_bf16(v, dtype) for k, v in layer.items()}


# ----------------------------------------------------------------- elementary ops

def rmsnorm(h, g, eps):
    """a = h * rsqrt(mean(h^2) + eps) * g, mean over the feature axis."""
    r = 1.0 / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + h.dtype.type(eps))
    return h * r * g


def layernorm(h, g, b, eps):
    """a = (h - mean) * rsqrt(var + eps) * g + b with the biased variance."""
    mu = np.mean(h, axis=-1, keepdims=True)
    c = h - mu
    var = np.mean(c * c, axis=-1, keepdims=True)
    return c / np.sqrt(var + h.dtype.type(eps)) * g + b


def linear(x, w, b=None):
    """y = x W^T (+ b), W stored [out, in]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu(x):
    """Exact GELU: 0.5 x (1 + erf(x / sqrt 2))."""
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0))).astype(x.dtype)


def softmax_rows(s):
    """Row softmax; -inf entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_probs(q, k, shape: StackShape):
    """Attention weights per (batch item, query head).

    q [S, Hq, hd], k [S, Hkv, hd] for ONE batch item -> P [Hq, S, S].
    Query head j reads key/value head j // (Hq // Hkv).  Causal: query i sees
    keys j <= i.
    """
    S = q.shape[0]
    grp = shape.n_q_heads // shape.n_kv_heads
    scale = q.dtype.type(1.0 / math.sqrt(shape.head_dim))
    kx = np.repeat(k, grp, axis=1)                       # [S, Hq, hd]
    s = np.einsum("ihd,jhd->hij", q, kx) * scale         # [Hq, S, S]
    if shape.causal:
        i = np.arange(S)[:, None]
        j = np.arange(S)[None, :]
        s = np.where(j <= i, s, -np.inf).astype(q.dtype)
    return softmax_rows(s)


def attention(q, k, v, B, S, shape: StackShape, operands=None):
    """softmax(q k^T / sqrt(hd) + mask) v.  q [B*S, Hq*hd], k/v [B*S, Hkv*hd] -> [B*S, Hq*hd]."""
    Hq, Hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    grp = Hq // Hkv
    out = np.empty((B * S, Hq * hd), dtype=q.dtype)
    for b in range(B):
        sl = slice(b * S, (b + 1) * S)
        qb = q[sl].reshape(S, Hq, hd)
        kb = k[sl].reshape(S, Hkv, hd)
        vb = v[sl].reshape(S, Hkv, hd)
        p = _operand(attention_probs(qb, kb, shape), operands)
        vx = np.repeat(vb, grp, axis=1)
        out[sl] = np.einsum("hij,jhd->ihd", p, vx).reshape(S, Hq * hd)
    return out


def mse_loss(y, t):
    """mean over every element of (y - t)^2."""
    d = (y - t).astype(np.float64)
    return float(np.mean(d * d))


# ----------------------------------------------------------------- layer forward

def _split_qkv(qkv, shape):
    nq = shape.n_q_heads * shape.head_dim
    nk = shape.n_kv_heads * shape.head_dim
    return qkv[:, :nq], qkv[:, nq:nq + nk], qkv[:, nq + nk:nq + 2 * nk]


def layer_forward(h, w, B, S, shape: StackShape, keep=False, operands=None):
    """One layer.  h [B*S, d].  Returns h_out (and the intermediates if keep).
    operands: None = nothing is rounded; "bf16" = the contractions' operands are (module header)."""
    eps = shape.norm_eps
    f = shape.d_ffn
    c = {"h0": h}
    rnd = lambda t: _operand(t, operands)
    if shape.arch == DECODER:
        a = rnd(rmsnorm(h, w["g1"], eps))
        qkv = rnd(linear(a, w["wqkv"]))
        q, k, v = _split_qkv(qkv, shape)
        o = rnd(attention(q, k, v, B, S, shape, operands))
        h1 = h + linear(o, w["wo"])
        m = rnd(rmsnorm(h1, w["g2"], eps))
        gu = linear(m, w["wgu"])
        g, u = gu[:, :f], gu[:, f:]
        z = rnd(silu(g) * u)
        h2 = h1 + linear(z, w["wd"])
        if keep:
            c.update(a=a, q=q, k=k, v=v, o=o, h1=h1, m=m, g=g, u=u, z=z)
    elif shape.arch == ENCODER:
        a = rnd(layernorm(h, w["ln1_g"], w["ln1_b"], eps))
        qkv = rnd(linear(a, w["wqkv"], w["bqkv"]))
        q, k, v = _split_qkv(qkv, shape)
        o = rnd(attention(q, k, v, B, S, shape, operands))
        h1 = h + linear(o, w["wo"], w["bo"])
        m = rnd(layernorm(h1, w["ln2_g"], w["ln2_b"], eps))
        u = linear(m, w["w1"], w["b1"])
        z = rnd(gelu(u))
        h2 = h1 + linear(z, w["w2"], w["b2"])
        if keep:
            c.update(a=a, q=q, k=k, v=v, o=o, h1=h1, m=m, u=u, z=z)
    else:
        raise ValueError(shape.arch)
    return (h2, c) if keep else h2


def stack_forward(x, layers, B, S, shape: StackShape, dtype=np.float32, n_layers=None, operands=None):
    """y = layer_{L-1}(... layer_0(x)).  x [B, S, d] or [B*S, d]; returns [B*S, d]."""
    h = np.asarray(x).reshape(B * S, shape.d_model).astype(dtype)
    L = shape.n_layers if n_layers is None else n_layers
    for l in range(L):
        h = layer_forward(h, _weights(layers[l], dtype), B, S, shape, operands=operands)
    return h


# ----------------------------------------------------------------- layer backward

def _rmsnorm_bwd(da, h, g, eps):
    d = h.shape[-1]
    r = 1.0 / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + h.dtype.type(eps))
    dg = np.sum(da * h * r, axis=0)
    dag = da * g
    dh = r * dag - h * (r ** 3) * (np.sum(dag * h, axis=-1, keepdims=True) / d)
    return dh, dg


def _layernorm_bwd(da, h, g, eps):
    mu = np.mean(h, axis=-1, keepdims=True)
    c = h - mu
    var = np.mean(c * c, axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(var + h.dtype.type(eps))
    xh = c * r
    dg = np.sum(da * xh, axis=0)
    db = np.sum(da, axis=0)
    dxh = da * g
    dh = r * (dxh - np.mean(dxh, axis=-1, keepdims=True)
              - xh * np.mean(dxh * xh, axis=-1, keepdims=True))
    return dh, dg, db


def _swiglu_bwd(dz, g, u):
    """z = silu(g) * u  ->  dg = dz u silu'(g), du = dz silu(g); silu'(g) = s (1 + g (1 - s)), s = sigmoid(g)."""
    s = 1.0 / (1.0 + np.exp(-g))
    return dz * u * (s * (1.0 + g * (1.0 - s))), dz * (g * s)


def _linear_bwd(dy, x, w):
    """y = x W^T + b  ->  dx = dy W, dW = dy^T x, db = column sums of dy."""
    return dy @ w, dy.T @ x, np.sum(dy, axis=0)


def _attention_bwd(do, q, k, v, B, S, shape):
    Hq, Hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    grp = Hq // Hkv
    scale = q.dtype.type(1.0 / math.sqrt(hd))
    dq = np.empty_like(q)
    dk = np.empty_like(k)
    dv = np.empty_like(v)
    for b in range(B):
        sl = slice(b * S, (b + 1) * S)
        qb = q[sl].reshape(S, Hq, hd)
        kb = k[sl].reshape(S, Hkv, hd)
        vb = v[sl].reshape(S, Hkv, hd)
        dob = do[sl].reshape(S, Hq, hd)
        p = attention_probs(qb, kb, shape)                       # [Hq, S, S]
        kx = np.repeat(kb, grp, axis=1)
        vx = np.repeat(vb, grp, axis=1)
        dvx = np.einsum("hij,ihd->jhd", p, dob)                  # P^T dO
        dp = np.einsum("ihd,jhd->hij", dob, vx)                  # dO V^T
        ds = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))   # softmax Jacobian
        dqb = np.einsum("hij,jhd->ihd", ds, kx) * scale
        dkx = np.einsum("hij,ihd->jhd", ds, qb) * scale
        dq[sl] = dqb.reshape(S, Hq * hd)
        dk[sl] = dkx.reshape(S, Hkv, grp, hd).sum(axis=2).reshape(S, Hkv * hd)
        dv[sl] = dvx.reshape(S, Hkv, grp, hd).sum(axis=2).reshape(S, Hkv * hd)
    return dq, dk, dv


def layer_backward(dh2, c, w, B, S, shape: StackShape):
    """Gradient of one layer.  Returns (dh_in, {name: dW})."""
    eps = shape.norm_eps
    gr = {}
    if shape.arch == DECODER:
        dz, gr["wd"], _ = _linear_bwd(dh2, c["z"], w["wd"])
        dg, du = _swiglu_bwd(dz, c["g"], c["u"])
        dgu = np.concatenate([dg, du], axis=1)
        dm, gr["wgu"], _ = _linear_bwd(dgu, c["m"], w["wgu"])
        dh1n, gr["g2"] = _rmsnorm_bwd(dm, c["h1"], w["g2"], eps)
        dh1 = dh2 + dh1n
        do, gr["wo"], _ = _linear_bwd(dh1, c["o"], w["wo"])
        dq, dk, dv = _attention_bwd(do, c["q"], c["k"], c["v"], B, S, shape)
        dqkv = np.concatenate([dq, dk, dv], axis=1)
        da, gr["wqkv"], _ = _linear_bwd(dqkv, c["a"], w["wqkv"])
        dh0n, gr["g1"] = _rmsnorm_bwd(da, c["h0"], w["g1"], eps)
        return dh1 + dh0n, gr
    dz, gr["w2"], gr["b2"] = _linear_bwd(dh2, c["z"], w["w2"])
    u = c["u"]
    dgelu = 0.5 * (1.0 + _erf(u / math.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    du = dz * dgelu.astype(u.dtype)
    dm, gr["w1"], gr["b1"] = _linear_bwd(du, c["m"], w["w1"])
    dh1n, gr["ln2_g"], gr["ln2_b"] = _layernorm_bwd(dm, c["h1"], w["ln2_g"], eps)
    dh1 = dh2 + dh1n
    do, gr["wo"], gr["bo"] = _linear_bwd(dh1, c["o"], w["wo"])
    dq, dk, dv = _attention_bwd(do, c["q"], c["k"], c["v"], B, S, shape)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    da, gr["wqkv"], gr["bqkv"] = _linear_bwd(dqkv, c["a"], w["wqkv"])
    dh0n, gr["ln1_g"], gr["ln1_b"] = _layernorm_bwd(da, c["h0"], w["ln1_g"], eps)
    return dh1 + dh0n, gr


def stack_forward_backward(x, target, layers, B, S, shape: StackShape, dtype=np.float64):
    """loss = mean((y - target)^2); returns (y, loss, dx, [per-layer grad dicts])."""
    T, d = B * S, shape.d_model
    h = np.asarray(x).reshape(T, d).astype(dtype)
    t = np.asarray(target).reshape(T, d).astype(dtype)
    caches = []
    for l in range(shape.n_layers):
        h, c = layer_forward(h, _weights(layers[l], dtype), B, S, shape, keep=True)
        caches.append(c)
    y = h
    diff = y - t
    loss = float(np.mean(diff.astype(np.float64) ** 2))
    dh = (2.0 / (T * d)) * diff
    grads = [None] * shape.n_layers
    for l in reversed(range(shape.n_layers)):
        dh, grads[l] = layer_backward(dh, caches[l], _weights(layers[l], dtype), B, S, shape)
        caches[l] = None
    return y, loss, dh, grads
