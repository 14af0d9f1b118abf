"""The training step on the GPU (forward, MSE, backward with re-streamed
weights, fp32 gradients streamed to pinned host blobs) against the oracle's
analytic gradients, and bit-identity of loss / dx / gradients over window
settings (the paper's fidelity claim covers training too, Sec. 4.2.2)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import stack_oracle as O  # noqa: E402
from paper_2410_08791_amd import binding as sp  # noqa: E402
from paper_2410_08791_amd import synth  # noqa: E402
from tests.gpu_util import DEV, dev_f32, max_rel  # noqa: E402

TOL = 2e-2


class TrainCase:
    def __init__(self, w):
        self.w = w
        self.desc = sp.make_desc(w)
        self.blobs, self.views = sp.pinned_blobs(w, self.desc)
        self.x = synth.make_input(w, "x")
        self.t = synth.make_input(w, "target")
        self.xd, self.td = dev_f32(self.x), dev_f32(self.t)
        self.gbytes = sp.sp_layer_grad_bytes(C.byref(self.desc))

    def run(self, k, p, calls=1, want_y=True, target=None, budget_layers=None, flags=0, pinned=0, frozen=0,
            want_dx=True, delay_us=0):
        w = self.w
        eng = sp.Engine(self.desc, self.blobs, k, p, flags=sp.SP_FLAG_TRAINING | flags, budget_layers=budget_layers,
                        pinned=pinned, frozen=frozen, delay_us=delay_us)
        gblobs = [torch.zeros(self.gbytes, dtype=torch.uint8, pin_memory=True) for _ in range(w.n_layers)]
        y = torch.zeros_like(self.xd) if want_y else None
        dx = torch.zeros_like(self.xd)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        td = self.td if target is None else target
        for _ in range(calls):
            for g in gblobs:
                g.fill_(0xFF)
            eng.forward_backward(self.xd, td, y, loss, dx if want_dx else None, gblobs, w.batch, w.seq)
            eng.sync()
        st = eng.stats()
        grads = [{n: v.copy() for n, v in sp.grad_views(self.desc, g.numpy()).items()} for g in gblobs]
        out = dict(loss=float(loss.item()), dx=dx.cpu().numpy().reshape(w.tokens, -1),
                   y=y.cpu().numpy().reshape(w.tokens, -1) if want_y else None, grads=grads, stats=st)
        assert eng.destroy() == sp.SP_OK
        return out

    def oracle(self, dtype=np.float64):
        w = self.w
        sh = O.StackShape(w.arch, w.n_layers, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn,
                          w.causal, w.norm_eps)
        return O.stack_forward_backward(self.x, self.t, self.views, w.batch, w.seq, sh, dtype=dtype)


def check_against_oracle(got, ref, tag):
    y, loss, dx, grads = ref
    if got["y"] is not None:
        assert max_rel(got["y"], y) <= TOL
    assert abs(got["loss"] - loss) <= TOL * loss, (got["loss"], loss)
    e = max_rel(got["dx"], dx.reshape(got["dx"].shape))
    worst = ("dx", e)
    assert e <= TOL, ("dx", e)
    for l, (gl, rl) in enumerate(zip(got["grads"], grads)):
        for n, r in rl.items():
            g = gl[n].reshape(r.shape)
            assert np.all(np.isfinite(g)), (l, n)
            e = max_rel(g, r)
            if e > worst[1]:
                worst = (f"layer {l} {n}", e)
            assert e <= TOL, (tag, l, n, e)
    print(f"{tag}: loss {got['loss']:.6f} vs {loss:.6f}; worst gradient error {worst[0]} = {worst[1]:.3e}")


@pytest.fixture(scope="module")
def small():
    return TrainCase(synth.Workload("train_small", "decoder", 3, 256, 4, 4, 64, 512, True, 2, 96, training=True))


def test_training_step_matches_oracle(small):
    got = small.run(2, 1)
    check_against_oracle(got, small.oracle(), "train_small")
    st = got["stats"]
    assert st.d2h_copies == 3 and st.d2h_bytes == 3 * small.gbytes
    assert st.h2d_copies == 3          # 3 layers, 3 slots: each layer crosses the link once


def test_training_bits_do_not_depend_on_the_window(small):
    base = small.run(8, 8)             # resident
    assert base["stats"].plan.fully_resident
    for k, p in [(1, 1), (2, 1), (1, 2)]:
        for bl in (None, 1):
            got = small.run(k, p, budget_layers=bl)
            assert got["loss"] == base["loss"], (k, p, bl)
            assert np.array_equal(got["dx"], base["dx"]) and np.array_equal(got["y"], base["y"]), (k, p, bl)
            for gl, bl_ in zip(got["grads"], base["grads"]):
                for n in gl:
                    assert np.array_equal(gl[n], bl_[n]), (k, p, n)


def test_training_repeated_calls_and_link_traffic():
    # 6 layers, 2 slots: forward copies 6, the turn re-uses 2, backward copies 4; the next
    # call finds layers 0,1 resident
    w = synth.Workload("train_l6", "decoder", 6, 256, 4, 2, 64, 512, True, 1, 128, training=True)
    c = TrainCase(w)
    a = c.run(1, 1, calls=1)
    b = c.run(1, 1, calls=3)
    assert a["loss"] == b["loss"] and np.array_equal(a["dx"], b["dx"])
    assert a["stats"].h2d_copies == 6 + 4
    assert b["stats"].h2d_copies == 10 + 2 * 8 and b["stats"].last_h2d_copies == 8
    check_against_oracle(b, c.oracle(), "train_l6 (grouped-query heads)")
    # two pinned layers next to the 2-slot ring: they are copied once in the handle's life, the
    # other four stream: 4 in the first forward, 2 in each backward and each later forward
    d = c.run(1, 1, calls=3, pinned=2)
    assert d["stats"].plan.n_pinned == 2 and d["stats"].plan.n_slots == 4
    assert d["stats"].h2d_copies == 2 + 4 + 2 + 2 * 4 and d["stats"].last_h2d_copies == 4
    assert d["loss"] == b["loss"] and np.array_equal(d["dx"], b["dx"])
    for gl, bl in zip(d["grads"], b["grads"]):
        for n in gl:
            assert np.array_equal(gl[n], bl[n]), n


def test_frozen_lower_layers():
    """The paper's 'half of layers frozen' rows (Table 2): the trainable layers' gradients
    are bit for bit those of the fully trainable run, frozen layers' gradient blobs are
    not written, and without an input gradient the backward stops above the frozen
    layers (fewer layer copies, fewer gradient copies)."""
    w = synth.Workload("train_l6", "decoder", 6, 256, 4, 2, 64, 512, True, 1, 128, training=True)
    c = TrainCase(w)
    full = c.run(1, 1, calls=2)
    for flags in (0, sp.SP_FLAG_KEEP_ACTIVATIONS):
        with_dx = c.run(1, 1, calls=2, frozen=3, flags=flags)
        no_dx = c.run(1, 1, calls=2, frozen=3, want_dx=False, flags=flags)
        for got in (with_dx, no_dx):
            assert got["loss"] == full["loss"] and np.array_equal(got["y"], full["y"])
            for l in range(6):
                for n, g in got["grads"][l].items():
                    if l >= 3:
                        assert np.array_equal(g, full["grads"][l][n]), (l, n)
                    else:
                        assert np.all(g.view(np.uint32) == 0xFFFFFFFF), (l, n)     # untouched fill
            assert got["stats"].d2h_copies == 2 * 3
        assert np.array_equal(with_dx["dx"], full["dx"])
        # forward 6 copies; the backward re-uses the 2 resident layers and stops at layer 3
        assert no_dx["stats"].h2d_copies < with_dx["stats"].h2d_copies
        ops = sp.trace_schedule(6, 2, 1, training=True, passes=4, frozen=3)
        assert no_dx["stats"].h2d_copies == sum(1 for o in ops if o[0] == 0)
    # everything frozen, no dx: forward and loss only
    none = c.run(1, 1, frozen=6, want_dx=False)
    assert none["loss"] == full["loss"] and none["stats"].d2h_copies == 0
    for bad in (-1, 7):
        with pytest.raises(sp.SuperpipeError):
            c.run(1, 1, frozen=bad)


def test_training_ragged_token_count_and_no_y():
    # T = 3*77 = 231 tokens: not a multiple of the 64-token contraction tile
    w = synth.Workload("train_ragged", "decoder", 2, 256, 2, 2, 128, 576, True, 3, 77, training=True)
    c = TrainCase(w)
    got = c.run(1, 1, want_y=False, calls=2)
    check_against_oracle(got, c.oracle(), "train_ragged")


def test_kept_activations_give_the_same_bits_as_recompute(small):
    """Without recompute (every layer's activations kept in HBM, the paper's 'without gradient
    checkpointing' column) the backward sees exactly the tensors the recompute would rebuild."""
    base = small.run(2, 1, calls=2)
    kept = small.run(2, 1, calls=2, flags=sp.SP_FLAG_KEEP_ACTIVATIONS)
    assert kept["loss"] == base["loss"] and np.array_equal(kept["dx"], base["dx"])
    for gl, bl in zip(kept["grads"], base["grads"]):
        for n in gl:
            assert np.array_equal(gl[n], bl[n]), n
    assert kept["stats"].plan.workspace_bytes > base["stats"].plan.workspace_bytes
    # ragged token count: the padded rows of every layer's set must read as zero
    w = synth.Workload("train_ragged_keep", "decoder", 3, 256, 2, 2, 128, 576, True, 3, 77, training=True)
    c = TrainCase(w)
    got = c.run(1, 1, flags=sp.SP_FLAG_KEEP_ACTIVATIONS, calls=2)
    check_against_oracle(got, c.oracle(), "train_ragged_keep")


def test_zero_loss_gives_zero_gradients(small):
    first = small.run(2, 1)
    y = dev_f32(first["y"].reshape(small.x.shape))
    got = small.run(2, 1, target=y)
    assert got["loss"] == 0.0 and not got["dx"].any()
    assert all(not g.any() for gl in got["grads"] for g in gl.values())


def test_pageable_gradient_buffers_are_refused(small):
    """Gradient blobs must be pinned: from pageable memory the device-to-host copies would block
    the host and lose their overlap with the backward pass."""
    w = small.w
    eng = sp.Engine(small.desc, small.blobs, 1, 1, flags=sp.SP_FLAG_TRAINING)
    good = [torch.zeros(small.gbytes, dtype=torch.uint8, pin_memory=True) for _ in range(w.n_layers)]
    bad = list(good)
    bad[1] = torch.zeros(small.gbytes, dtype=torch.uint8)          # pageable
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    with pytest.raises(sp.SuperpipeError) as ei:
        eng.forward_backward(small.xd, small.td, None, loss, None, bad, w.batch, w.seq)
    assert ei.value.code == sp.SP_ERR_NOT_PINNED
    # an argument error leaves the handle usable
    eng.forward_backward(small.xd, small.td, None, loss, None, good, w.batch, w.seq)
    eng.sync()
    assert np.isfinite(loss.item())
    assert eng.destroy() == sp.SP_OK


def test_training_with_injected_delays_gives_the_same_bits(small):
    base = small.run(8, 8)
    got = small.run(1, 1, calls=2, flags=sp.SP_FLAG_DELAY | sp.SP_FLAG_POISON, delay_us=300)
    assert got["loss"] == base["loss"] and np.array_equal(got["dx"], base["dx"])
    for gl, bl in zip(got["grads"], base["grads"]):
        for n in gl:
            assert np.array_equal(gl[n], bl[n]), n


def test_forward_only_handle_refuses_training(small):
    eng = sp.Engine(small.desc, small.blobs, 1, 1)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    with pytest.raises(sp.SuperpipeError) as ei:
        eng.forward_backward(small.xd, small.td, None, loss, None, [], 2, 96)
    assert ei.value.code == sp.SP_ERR_STATE
    eng.destroy()


def test_train1p3b_layer_shape():
    """The training workload's layer shape (d 2048, 16 heads x 128, ffn 5504), two layers,
    2 x 1024 tokens so that the fp32 oracle's backward finishes in seconds."""
    w = synth.WORKLOADS["train1p3b"].with_(n_layers=2, batch=2)
    c = TrainCase(w)
    got = c.run(1, 1)
    check_against_oracle(got, c.oracle(np.float32), "train1p3b x2 layers, batch 2")


@pytest.mark.parametrize("hd,seq", [(64, 50), (80, 33)])
def test_encoder_training_matches_oracle(hd, seq):
    """The encoder layer kind (LayerNorm, biased linears, GELU, bidirectional attention) through
    the same training path: loss, dx and all twelve tensors' gradients per layer against the
    oracle; same bits for every window and with kept activations; frozen lower layer."""
    d = 4 * hd
    w = synth.Workload(f"train_enc{hd}", "encoder", 3, d, 4, 4, hd, 4 * d, False, 2, seq, training=True)
    c = TrainCase(w)
    base = c.run(1, 1, calls=2)
    check_against_oracle(base, c.oracle(), w.name)
    for kwargs in (dict(k=4, p=4), dict(k=1, p=1, flags=sp.SP_FLAG_KEEP_ACTIVATIONS), dict(k=1, p=1, pinned=1)):
        k, p = kwargs.pop("k"), kwargs.pop("p")
        got = c.run(k, p, calls=2, **kwargs)
        assert got["loss"] == base["loss"] and np.array_equal(got["dx"], base["dx"])
        for gl, bl in zip(got["grads"], base["grads"]):
            for n in gl:
                assert np.array_equal(gl[n], bl[n]), (kwargs, n)
    fr = c.run(1, 1, frozen=1)
    assert np.array_equal(fr["dx"], base["dx"])
    for n, g in fr["grads"][2].items():
        assert np.array_equal(g, base["grads"][2][n]), n
    assert all(np.all(g.view(np.uint32) == 0xFFFFFFFF) for g in fr["grads"][0].values())


def test_vith_layer_shape_training():
    """ViT-H layer shape (d 1280, 16 heads of 80, ffn 5120), two layers, 4 images of 257 tokens."""
    w = synth.WORKLOADS["vith"].with_(n_layers=2, batch=4, training=True)
    c = TrainCase(w)
    got = c.run(1, 1)
    check_against_oracle(got, c.oracle(np.float32), "vith x2 layers, batch 4 (fp32 oracle)")


def _host_update(views_l, grads_l):
    """A host 'optimizer' for the loop test: w <- bf16(w - 0.01 * g / max|g|) per tensor, so that
    every tensor moves by about half its own spread whatever the gradient's scale."""
    for n, v in views_l.items():
        g = grads_l[n].reshape(v.shape)
        m = float(np.abs(g).max())
        if m > 0:
            v[...] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(v) - np.float32(0.01 / m) * g)


@pytest.mark.parametrize("k,p,pinned,budget_layers", [(8, 8, 0, None), (1, 1, 1, None), (1, 1, 0, 1)])
def test_training_loop_with_host_updates_between_steps(small, k, p, pinned, budget_layers):
    """Two steps with the host rewriting the weights in between.  Each layer is updated as soon
    as its own gradient has landed (from the last layer down) and the handle is told; the second
    step must run on the new weights: bit for bit what a fresh handle computes from them, and
    within the tolerance of the oracle on them.  The resident window (first case) is where stale
    weights would otherwise stay in use."""
    w, desc = small.w, small.desc
    blobs, views = sp.pinned_blobs(w, desc)              # private weights: this test rewrites them
    L = w.n_layers

    def step(eng):
        gblobs = [torch.full((small.gbytes,), 0xFF, dtype=torch.uint8).pin_memory() for _ in range(L)]
        y, dx = torch.zeros_like(small.xd), torch.zeros_like(small.xd)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        eng.forward_backward(small.xd, small.td, y, loss, dx, gblobs, w.batch, w.seq)
        return gblobs, y, dx, loss

    def collect(eng, gblobs, y, dx, loss):
        eng.sync()
        return dict(loss=float(loss.item()), dx=dx.cpu().numpy().reshape(w.tokens, -1),
                    y=y.cpu().numpy().reshape(w.tokens, -1),
                    grads=[{n: v.copy() for n, v in sp.grad_views(desc, g.numpy()).items()} for g in gblobs])

    eng = sp.Engine(desc, blobs, k, p, flags=sp.SP_FLAG_TRAINING, pinned=pinned, budget_layers=budget_layers)
    with pytest.raises(sp.SuperpipeError):
        eng.wait_gradient(0)                             # no step yet
    out = step(eng)
    for l in reversed(range(L)):
        eng.wait_gradient(l)
        _host_update(views[l], sp.grad_views(desc, out[0][l].numpy()))
        eng.weights_updated(l)
    first = collect(eng, *out)
    second = collect(eng, *step(eng))
    with pytest.raises(sp.SuperpipeError):
        eng.wait_gradient(L)
    assert eng.destroy() == sp.SP_OK
    assert not np.array_equal(first["y"], second["y"]) and second["loss"] != first["loss"]

    fresh = sp.Engine(desc, blobs, 1, 2, flags=sp.SP_FLAG_TRAINING)
    ref = collect(fresh, *step(fresh))
    assert fresh.destroy() == sp.SP_OK
    assert second["loss"] == ref["loss"]
    assert np.array_equal(second["y"], ref["y"]) and np.array_equal(second["dx"], ref["dx"])
    for gl, rl in zip(second["grads"], ref["grads"]):
        for n in gl:
            assert np.array_equal(gl[n], rl[n]), n
    sh = O.StackShape(w.arch, L, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn, w.causal, w.norm_eps)
    check_against_oracle(second, O.stack_forward_backward(small.x, small.t, views, w.batch, w.seq, sh),
                         f"second step after host updates (k={k}, p={p}, pinned={pinned})")


def test_wait_gradient_refuses_frozen_layers_and_forward_handles(small):
    w, desc = small.w, small.desc
    eng = sp.Engine(desc, small.blobs, 1, 1, flags=sp.SP_FLAG_TRAINING, frozen=1)
    gblobs = [torch.zeros(small.gbytes, dtype=torch.uint8, pin_memory=True) for _ in range(w.n_layers)]
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    eng.forward_backward(small.xd, small.td, None, loss, None, gblobs, w.batch, w.seq)
    eng.wait_gradient(w.n_layers - 1)
    eng.wait_gradient(1)
    with pytest.raises(sp.SuperpipeError) as ei:
        eng.wait_gradient(0)
    assert ei.value.code == sp.SP_ERR_STATE
    eng.sync()
    assert eng.destroy() == sp.SP_OK
    fwd = sp.Engine(desc, small.blobs, 1, 1)
    with pytest.raises(sp.SuperpipeError) as ei:
        fwd.wait_gradient(0)
    assert ei.value.code == sp.SP_ERR_STATE
    assert fwd.destroy() == sp.SP_OK
