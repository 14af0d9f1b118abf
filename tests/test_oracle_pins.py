"""Pins for oracle/stack_oracle.py: each oracle function is checked against
something other than itself -- scalar-loop definitions written out here in
plain Python floats, closed forms, textbook values, invariants and central
finite differences.  CPU only."""
import math

import numpy as np
import pytest

from oracle import stack_oracle as O

RNG = np.random.default_rng(1234)


# ------------------------------------------------------------------ scalar-loop definitions
def bf_rmsnorm(h, g, eps):
    out = [[0.0] * len(h[0]) for _ in h]
    for t, row in enumerate(h):
        ms = sum(v * v for v in row) / len(row)
        r = 1.0 / math.sqrt(ms + eps)
        for i, v in enumerate(row):
            out[t][i] = v * r * g[i]
    return out


def bf_layernorm(h, g, b, eps):
    out = [[0.0] * len(h[0]) for _ in h]
    for t, row in enumerate(h):
        n = len(row)
        mu = sum(row) / n
        var = sum((v - mu) ** 2 for v in row) / n
        r = 1.0 / math.sqrt(var + eps)
        for i, v in enumerate(row):
            out[t][i] = (v - mu) * r * g[i] + b[i]
    return out


def bf_linear(x, w, b=None):
    # y[t][o] = sum_i x[t][i] * w[o][i] + b[o]
    out = []
    for row in x:
        out.append([sum(row[i] * w[o][i] for i in range(len(row))) + (b[o] if b is not None else 0.0)
                    for o in range(len(w))])
    return out


def bf_round(x):
    """Scalar nearest-bfloat16, ties to even, through the float32 bit pattern (struct, no numpy)."""
    import struct
    u = struct.unpack("<I", struct.pack("<f", x))[0]
    top, rem = u >> 16, u & 0xFFFF
    if rem > 0x8000 or (rem == 0x8000 and top & 1):
        top += 1
    return struct.unpack("<f", struct.pack("<I", (top << 16) & 0xFFFFFFFF))[0]


def ident(x):
    return x


def rows(rnd, m):
    return [[rnd(x) for x in r] for r in m]


def bf_attention(q, k, v, B, S, Hq, Hkv, hd, causal, rnd=ident):
    T = B * S
    out = [[0.0] * (Hq * hd) for _ in range(T)]
    grp = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            kvh = h // grp
            for i in range(S):
                keys = range(i + 1) if causal else range(S)
                sc = []
                for j in keys:
                    s = 0.0
                    for e in range(hd):
                        s += q[b * S + i][h * hd + e] * k[b * S + j][kvh * hd + e]
                    sc.append(s / math.sqrt(hd))
                mx = max(sc)
                ex = [math.exp(s - mx) for s in sc]
                den = sum(ex)
                for e in range(hd):
                    acc = 0.0
                    for jj, j in enumerate(keys):
                        acc += rnd(ex[jj] / den) * v[b * S + j][kvh * hd + e]
                    out[b * S + i][h * hd + e] = acc
    return out


def bf_decoder_layer(h, w, B, S, sh, rnd=ident):
    d, f = sh.d_model, sh.d_ffn
    nq, nk = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim
    a = rows(rnd, bf_rmsnorm(h, w["g1"], sh.norm_eps))
    qkv = rows(rnd, bf_linear(a, w["wqkv"]))
    q = [r[:nq] for r in qkv]
    k = [r[nq:nq + nk] for r in qkv]
    v = [r[nq + nk:] for r in qkv]
    o = rows(rnd, bf_attention(q, k, v, B, S, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.causal, rnd))
    ow = bf_linear(o, w["wo"])
    h1 = [[h[t][i] + ow[t][i] for i in range(d)] for t in range(len(h))]
    m = rows(rnd, bf_rmsnorm(h1, w["g2"], sh.norm_eps))
    gu = bf_linear(m, w["wgu"])
    z = [[rnd((r[j] / (1.0 + math.exp(-r[j]))) * r[f + j]) for j in range(f)] for r in gu]
    zw = bf_linear(z, w["wd"])
    return [[h1[t][i] + zw[t][i] for i in range(d)] for t in range(len(h))]


def bf_encoder_layer(h, w, B, S, sh, rnd=ident):
    d = sh.d_model
    nq, nk = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim
    a = rows(rnd, bf_layernorm(h, w["ln1_g"], w["ln1_b"], sh.norm_eps))
    qkv = rows(rnd, bf_linear(a, w["wqkv"], w["bqkv"]))
    q = [r[:nq] for r in qkv]
    k = [r[nq:nq + nk] for r in qkv]
    v = [r[nq + nk:] for r in qkv]
    o = rows(rnd, bf_attention(q, k, v, B, S, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, False, rnd))
    ow = bf_linear(o, w["wo"], w["bo"])
    h1 = [[h[t][i] + ow[t][i] for i in range(d)] for t in range(len(h))]
    m = rows(rnd, bf_layernorm(h1, w["ln2_g"], w["ln2_b"], sh.norm_eps))
    u = bf_linear(m, w["w1"], w["b1"])
    z = [[rnd(0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))) for x in r] for r in u]
    zw = bf_linear(z, w["w2"], w["b2"])
    return [[h1[t][i] + zw[t][i] for i in range(d)] for t in range(len(h))]


# ------------------------------------------------------------------ helpers
def small_shape(arch, causal=True, Hq=4, Hkv=2, hd=3, d=10, f=7, L=2):
    return O.StackShape(arch, L, d, Hq, Hkv, hd, f, causal, 1e-5)


def rand_layer(sh, scale=0.3):
    d, f = sh.d_model, sh.d_ffn
    nq, nk = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim
    r = lambda *s: RNG.standard_normal(s) * scale
    if sh.arch == O.DECODER:
        return dict(g1=1 + r(d), wqkv=r(nq + 2 * nk, d), wo=r(d, nq), g2=1 + r(d),
                    wgu=r(2 * f, d), wd=r(d, f))
    return dict(ln1_g=1 + r(d), ln1_b=r(d), wqkv=r(nq + 2 * nk, d), bqkv=r(nq + 2 * nk),
                wo=r(d, nq), bo=r(d), ln2_g=1 + r(d), ln2_b=r(d),
                w1=r(f, d), b1=r(f), w2=r(d, f), b2=r(d))


def tolist(w):
    return {k: v.tolist() for k, v in w.items()}


# ------------------------------------------------------------------ elementary ops
def test_decode_bf16_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x3DCC, 0x0000, 0x8000, 0x7F7F], dtype=np.uint16)
    got = O.decode_bf16(bits, np.float64)
    want = [1.0, -2.0, 0.099609375, 0.0, -0.0, 3.3895313892515355e38]
    assert got.tolist() == want
    assert math.copysign(1.0, got[4]) == -1.0


def test_rmsnorm_vs_loops_and_closed_form():
    h = RNG.standard_normal((5, 9))
    g = 1 + 0.1 * RNG.standard_normal(9)
    np.testing.assert_allclose(O.rmsnorm(h, g, 1e-5), bf_rmsnorm(h.tolist(), g.tolist(), 1e-5), rtol=1e-13)
    # unit gain, eps = 0: every row has mean square exactly 1
    a = O.rmsnorm(h, np.ones(9), 0.0)
    np.testing.assert_allclose(np.mean(a * a, axis=-1), 1.0, rtol=1e-13)
    # eps matters: a row of zeros maps to zeros, not NaN
    assert np.all(O.rmsnorm(np.zeros((1, 9)), g, 1e-5) == 0.0)


def test_layernorm_vs_loops_and_moments():
    h = RNG.standard_normal((4, 11)) * 3 + 2
    g = 1 + 0.1 * RNG.standard_normal(11)
    b = 0.1 * RNG.standard_normal(11)
    np.testing.assert_allclose(O.layernorm(h, g, b, 1e-5),
                               bf_layernorm(h.tolist(), g.tolist(), b.tolist(), 1e-5), rtol=1e-12)
    a = O.layernorm(h, np.ones(11), np.zeros(11), 0.0)
    np.testing.assert_allclose(a.mean(-1), 0.0, atol=1e-14)
    np.testing.assert_allclose(a.var(-1), 1.0, rtol=1e-12)   # biased variance


def test_linear_is_x_times_w_transposed():
    x = RNG.standard_normal((3, 5))
    w = RNG.standard_normal((4, 5))
    b = RNG.standard_normal(4)
    np.testing.assert_allclose(O.linear(x, w, b), bf_linear(x.tolist(), w.tolist(), b.tolist()), rtol=1e-13)
    # a one-hot weight row picks one input feature
    w0 = np.zeros((4, 5)); w0[2, 3] = 1.0
    y = O.linear(x, w0)
    assert np.array_equal(y[:, 2], x[:, 3]) and np.all(y[:, [0, 1, 3]] == 0)


def test_activation_textbook_values():
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(np.array([1.0, -1.0])), [0.7310585786300049, -0.2689414213699951], rtol=1e-15)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    # gelu(1) = Phi(1); gelu(-x) = gelu(x) - x
    np.testing.assert_allclose(O.gelu(np.array([1.0]))[0], 0.8413447460685429, rtol=1e-14)
    x = RNG.standard_normal(7)
    np.testing.assert_allclose(O.gelu(-x), O.gelu(x) - x, atol=1e-15)


def test_softmax_rows():
    s = RNG.standard_normal((3, 6))
    s[1, 4:] = -np.inf
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-14)
    assert np.all(p[1, 4:] == 0.0)
    np.testing.assert_allclose(O.softmax_rows(np.zeros((1, 4))), 0.25)
    # shift invariance
    np.testing.assert_allclose(O.softmax_rows(s + 100.0), p, rtol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_attention_vs_loops(causal, Hq, Hkv):
    B, S, hd = 2, 5, 3
    sh = O.StackShape(O.DECODER, 1, Hq * hd, Hq, Hkv, hd, 4, causal)
    q = RNG.standard_normal((B * S, Hq * hd))
    k = RNG.standard_normal((B * S, Hkv * hd))
    v = RNG.standard_normal((B * S, Hkv * hd))
    got = O.attention(q, k, v, B, S, sh)
    want = bf_attention(q.tolist(), k.tolist(), v.tolist(), B, S, Hq, Hkv, hd, causal)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_attention_special_cases():
    B, S, Hq, hd = 1, 6, 2, 4
    sh = O.StackShape(O.DECODER, 1, Hq * hd, Hq, Hq, hd, 4, True)
    q = RNG.standard_normal((S, Hq * hd)); k = RNG.standard_normal((S, Hq * hd)); v = RNG.standard_normal((S, Hq * hd))
    o = O.attention(q, k, v, B, S, sh)
    # causal: the first query sees only the first key
    np.testing.assert_allclose(o[0], v[0], rtol=1e-14)
    # zero queries -> uniform weights -> running mean of v (causal) / plain mean (bidirectional)
    o0 = O.attention(np.zeros_like(q), k, v, B, S, sh)
    np.testing.assert_allclose(o0, np.cumsum(v, 0) / np.arange(1, S + 1)[:, None], rtol=1e-13)
    shb = O.StackShape(O.ENCODER, 1, Hq * hd, Hq, Hq, hd, 4, False)
    ob = O.attention(np.zeros_like(q), k, v, B, S, shb)
    np.testing.assert_allclose(ob, np.broadcast_to(v.mean(0), v.shape), rtol=1e-13)
    # grouped-query heads == multi-head with the kv heads written out per query head
    Hkv = 1
    shg = O.StackShape(O.DECODER, 1, Hq * hd, Hq, Hkv, hd, 4, True)
    kg = RNG.standard_normal((S, Hkv * hd)); vg = RNG.standard_normal((S, Hkv * hd))
    og = O.attention(q, kg, vg, B, S, shg)
    om = O.attention(q, np.tile(kg, (1, Hq)), np.tile(vg, (1, Hq)), B, S, sh)
    np.testing.assert_allclose(og, om, rtol=1e-14)


def test_round_bf16_known_patterns():
    """Nearest bfloat16, ties to even: values worked out by hand (spacing 2^-7 at 1.0)."""
    cases = [(1.0, 1.0), (1.0 + 2.0 ** -8, 1.0),                      # tie, lower neighbour even
             (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),                  # tie, upper neighbour even
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7),         # just above the tie
             (1.0 + 2.0 ** -8 - 2.0 ** -20, 1.0),                     # just below
             (-(1.0 + 3 * 2.0 ** -8), -(1.0 + 2.0 ** -6)), (0.0, 0.0),
             (0.1, 0.10009765625),                                    # 0x3DCD: 205 * 2^-11
             (3.0e38, 226 * 2.0 ** 120),                              # spacing 2^120 there: 225.7 -> 226
             (2.0 ** -130, 2.0 ** -130)]                              # a denormal with a bf16 pattern
    x = np.array([c[0] for c in cases])
    assert O.round_bf16(x).tolist() == [c[1] for c in cases]
    assert O.round_bf16(x.astype(np.float32)).dtype == np.float32
    assert [bf_round(c[0]) for c in cases] == [c[1] for c in cases]   # the scalar stand-in used below
    r = RNG.standard_normal(4096) * np.exp(RNG.uniform(-20, 20, 4096))
    q = O.round_bf16(r)
    assert np.array_equal(O.round_bf16(q), q)                          # idempotent
    assert np.all(np.abs(q - r) <= 2.0 ** -8 * np.abs(r) * (1 + 1e-6))  # half a step of 2^-7 at the bottom of a binade
    assert np.all((q.astype(np.float32).view(np.uint32) & 0xFFFF) == 0)


# ------------------------------------------------------------------ whole layer / stack
@pytest.mark.parametrize("arch", [O.DECODER, O.ENCODER])
def test_layer_with_bf16_operands_vs_scalar_composition(arch):
    """operands="bf16": the scalar-loop layer with the scalar rounding at the six operand points
    (normed activations twice, q/k/v, attention weights, attention output, activation output)."""
    B, S = 2, 4
    sh = small_shape(arch, causal=(arch == O.DECODER))
    w = rand_layer(sh)
    h = RNG.standard_normal((B * S, sh.d_model))
    got = O.layer_forward(h, w, B, S, sh, operands="bf16")
    bf = bf_decoder_layer if arch == O.DECODER else bf_encoder_layer
    want = bf(h.tolist(), tolist(w), B, S, sh, rnd=bf_round)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)
    plain = O.layer_forward(h, w, B, S, sh)
    dev = np.max(np.abs(got - plain)) / np.max(np.abs(plain - h))
    assert 1e-5 < dev < 2e-2, dev            # it does round, and by about what six roundings of 2^-9 give
    st = O.stack_forward(h, [w, w], B, S, sh, dtype=np.float64, operands="bf16")
    np.testing.assert_array_equal(st, O.layer_forward(got, w, B, S, sh, operands="bf16"))


@pytest.mark.parametrize("arch", [O.DECODER, O.ENCODER])
def test_layer_vs_scalar_composition(arch):
    B, S = 2, 4
    sh = small_shape(arch, causal=(arch == O.DECODER))
    w = rand_layer(sh)
    h = RNG.standard_normal((B * S, sh.d_model))
    got = O.layer_forward(h, w, B, S, sh)
    bf = bf_decoder_layer if arch == O.DECODER else bf_encoder_layer
    want = bf(h.tolist(), tolist(w), B, S, sh)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("arch", [O.DECODER, O.ENCODER])
def test_stack_is_composition_and_takes_bf16_bits(arch):
    B, S = 1, 3
    sh = small_shape(arch, causal=(arch == O.DECODER), L=3)
    # weights given as bf16 bit patterns must equal the same values given as floats
    layers_f, layers_b = [], []
    for _ in range(sh.n_layers):
        w = rand_layer(sh)
        bits = {k: (np.float32(v).view(np.uint32) >> 16).astype(np.uint16) for k, v in w.items()}
        layers_b.append(bits)
        layers_f.append({k: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64) for k, b in bits.items()})
    x = RNG.standard_normal((B, S, sh.d_model))
    y = O.stack_forward(x, layers_b, B, S, sh, dtype=np.float64)
    h = x.reshape(B * S, -1)
    bf = bf_decoder_layer if arch == O.DECODER else bf_encoder_layer
    hl = h.tolist()
    for w in layers_f:
        hl = bf(hl, tolist(w), B, S, sh)
    np.testing.assert_allclose(y, hl, rtol=1e-10, atol=1e-12)
    # n_layers argument runs a prefix
    y1 = O.stack_forward(x, layers_b, B, S, sh, dtype=np.float64, n_layers=1)
    np.testing.assert_allclose(y1, bf(h.tolist(), tolist(layers_f[0]), B, S, sh), rtol=1e-11, atol=1e-13)


def test_zero_output_projections_give_identity():
    B, S = 2, 3
    sh = small_shape(O.DECODER)
    layers = []
    for _ in range(sh.n_layers):
        w = rand_layer(sh)
        w["wo"][:] = 0.0
        w["wd"][:] = 0.0
        layers.append(w)
    x = RNG.standard_normal((B, S, sh.d_model))
    y = O.stack_forward(x, layers, B, S, sh, dtype=np.float64)
    assert np.array_equal(y, x.reshape(B * S, -1))


@pytest.mark.parametrize("arch", [O.DECODER, O.ENCODER])
def test_batch_items_are_independent(arch):
    B, S = 3, 4
    sh = small_shape(arch, causal=(arch == O.DECODER))
    layers = [rand_layer(sh) for _ in range(sh.n_layers)]
    x = RNG.standard_normal((B, S, sh.d_model))
    y = O.stack_forward(x, layers, B, S, sh, dtype=np.float64).reshape(B, S, -1)
    y1 = O.stack_forward(x[1:2], layers, 1, S, sh, dtype=np.float64).reshape(S, -1)
    np.testing.assert_allclose(y[1], y1, rtol=1e-12, atol=1e-14)


def test_causal_prefix_property():
    # with a causal mask, the first S' outputs do not depend on later tokens
    B, S = 1, 6
    sh = small_shape(O.DECODER, causal=True)
    layers = [rand_layer(sh) for _ in range(sh.n_layers)]
    x = RNG.standard_normal((B, S, sh.d_model))
    y = O.stack_forward(x, layers, B, S, sh, dtype=np.float64)
    y4 = O.stack_forward(x[:, :4], layers, B, 4, sh, dtype=np.float64)
    np.testing.assert_allclose(y[:4], y4, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ backward
def test_mse_closed_form():
    y = np.array([[1.0, 2.0], [3.0, 5.0]]); t = np.array([[0.0, 2.0], [1.0, 1.0]])
    assert O.mse_loss(y, t) == (1 + 0 + 4 + 16) / 4


@pytest.mark.parametrize("arch", [O.DECODER, O.ENCODER])
def test_backward_vs_central_differences(arch):
    B, S = 2, 3
    sh = small_shape(arch, causal=(arch == O.DECODER))
    layers = [rand_layer(sh) for _ in range(sh.n_layers)]
    x = RNG.standard_normal((B, S, sh.d_model))
    t = RNG.standard_normal((B, S, sh.d_model))
    y, loss, dx, grads = O.stack_forward_backward(x, t, layers, B, S, sh, dtype=np.float64)
    np.testing.assert_allclose(loss, O.mse_loss(O.stack_forward(x, layers, B, S, sh, dtype=np.float64),
                                                t.reshape(B * S, -1)), rtol=1e-14)

    def f():
        return O.mse_loss(O.stack_forward(x, layers, B, S, sh, dtype=np.float64), t.reshape(B * S, -1))

    eps = 1e-6
    pick = np.random.default_rng(7)

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + eps; fp = f()
        arr[idx] = old - eps; fm = f()
        arr[idx] = old
        return (fp - fm) / (2 * eps)

    scale = max(np.max(np.abs(g)) for gl in grads for g in gl.values())
    for l in range(sh.n_layers):
        assert set(grads[l]) == set(layers[l])
        for name, w in layers[l].items():
            assert grads[l][name].shape == w.shape
            for _ in range(4):
                idx = tuple(pick.integers(0, n) for n in w.shape)
                np.testing.assert_allclose(grads[l][name][idx], fd(w, idx), rtol=2e-6, atol=1e-8 * scale,
                                           err_msg=f"layer {l} {name}{idx}")
    dx = dx.reshape(x.shape)
    for _ in range(8):
        idx = tuple(pick.integers(0, n) for n in x.shape)
        np.testing.assert_allclose(dx[idx], fd(x, idx), rtol=2e-6, atol=1e-10)


def test_zero_loss_gives_zero_gradients():
    B, S = 1, 4
    sh = small_shape(O.DECODER)
    layers = [rand_layer(sh) for _ in range(sh.n_layers)]
    x = RNG.standard_normal((B, S, sh.d_model))
    y = O.stack_forward(x, layers, B, S, sh, dtype=np.float64)
    _, loss, dx, grads = O.stack_forward_backward(x, y, layers, B, S, sh, dtype=np.float64)
    assert loss == 0.0 and not dx.any()
    assert all(not g.any() for gl in grads for g in gl.values())


@pytest.mark.parametrize("arch,causal", [(O.DECODER, True), (O.ENCODER, False)])
def test_float32_mode_tracks_float64(arch, causal):
    """The float32 mode (the one the full-width GPU tests and the stored full-depth runs use) stays
    within float32 rounding of the float64 mode, forward and backward, for both layer kinds; the
    float64 mode is what the scalar-loop definitions and finite differences above pin."""
    B, S = 2, 8
    sh = small_shape(arch, d=16, f=24, Hq=4, Hkv=2 if arch == O.DECODER else 4, hd=4, causal=causal)
    layers = [rand_layer(sh) for _ in range(sh.n_layers)]
    x = RNG.standard_normal((B, S, sh.d_model))
    t = RNG.standard_normal((B, S, sh.d_model))
    y64 = O.stack_forward(x, layers, B, S, sh, dtype=np.float64)
    y32 = O.stack_forward(x, layers, B, S, sh, dtype=np.float32)
    assert y32.dtype == np.float32
    np.testing.assert_allclose(y32, y64, rtol=0, atol=2e-5 * np.max(np.abs(y64)))
    _, l64, dx64, g64 = O.stack_forward_backward(x, t, layers, B, S, sh, dtype=np.float64)
    _, l32, dx32, g32 = O.stack_forward_backward(x, t, layers, B, S, sh, dtype=np.float32)
    assert abs(l32 - l64) <= 1e-5 * l64
    np.testing.assert_allclose(dx32, dx64, rtol=0, atol=5e-5 * np.max(np.abs(dx64)))
    for a, b in zip(g32, g64):
        for n in b:
            np.testing.assert_allclose(a[n], b[n], rtol=0, atol=5e-5 * np.max(np.abs(b[n])) + 1e-12, err_msg=n)
