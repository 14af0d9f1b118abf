"""The schedule cost model and the window tuner (grid search over k and k', Sec. 4.2;
adaptive selection, Sec. 5), checked on the host against closed forms and against a
replay of the traced op list written here independently of the library's model."""
import ctypes as C
import random

import pytest

from paper_2410_08791_amd import binding as sp, synth

COPY, FWD, BWD = 0, 1, 2
GRAD_SLOTS = 4


def replay(ops, cost, training, calls_passes):
    """End-to-end times per call from the op list: three in-order streams."""
    copy_ms, fwd_ms, bwd_ms, grad_ms = cost
    t_copy = t_comp = t_grad = floor = 0.0
    loaded, done = {}, {}
    gfree = [0.0] * GRAD_SLOTS
    gs = 0
    out = []
    passes_per_call = 2 if training else 1
    begin = 0.0
    for i, (kind, layer, slot, wait, ps) in enumerate(ops):
        if i == 0 or ps != ops[i - 1][4]:
            if ps % passes_per_call == 0:
                if ps:
                    out.append((max(t_copy, t_comp, t_grad) if training else t_comp) - begin)
                begin = max(t_copy, t_comp, t_grad) if training else t_comp
                if training:
                    floor = begin
        if kind == COPY:
            b = max(t_copy, floor, done.get(wait, 0.0) if wait >= 0 else 0.0)
            t_copy = b + copy_ms
            loaded[layer] = t_copy
        else:
            b = max(t_comp, floor, loaded[layer] if wait else 0.0)
            if kind == FWD:
                t_comp = b + fwd_ms
            else:
                b = max(b, gfree[gs])
                t_comp = b + bwd_ms
                t_grad = max(t_grad, t_comp) + grad_ms
                gfree[gs] = t_grad
                gs = (gs + 1) % GRAD_SLOTS
            done[layer] = t_comp
    out.append((max(t_copy, t_comp, t_grad) if training else t_comp) - begin)
    return out


@pytest.mark.parametrize("training", [False, True])
def test_model_equals_replay_of_the_traced_schedule(training):
    rnd = random.Random(5 + training)
    for _ in range(200):
        L = rnd.randint(1, 24)
        n = rnd.randint(1, L)
        wrap = (not training) and rnd.random() < 0.5
        R = rnd.randint(0, n - 1) if n < L else 0
        p = rnd.randint(1, max(n - R - 1, 1))
        calls = rnd.randint(1, 4)
        cost = (rnd.uniform(0, 5), rnd.uniform(0.1, 5), rnd.uniform(0.1, 9), rnd.uniform(0, 6))
        ops = sp.trace_schedule(L, n, p, training=training, wrap=wrap, passes=calls * (2 if training else 1),
                                pinned=R)
        want = replay(ops, cost, training, calls)[-1]
        got = sp.simulate_call_ms(L, n, p, cost, training=training, wrap=wrap, calls=calls, pinned=R)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-12), (L, n, R, p, wrap, calls, cost)


def test_closed_forms_forward():
    L = 32
    # copy-bound, steady state with wrap-around prefetch: the link never idles
    assert sp.simulate_call_ms(L, 2, 1, (7.0, 1.0, 0, 0), wrap=True, calls=3) == pytest.approx(L * 7.0)
    # compute-bound, steady state: copies vanish behind compute
    assert sp.simulate_call_ms(L, 3, 1, (1.0, 4.0, 0, 0), wrap=True, calls=3) == pytest.approx(L * 4.0)
    # first call, compute-bound: only the first copy is exposed
    assert sp.simulate_call_ms(L, 2, 1, (1.0, 4.0, 0, 0), calls=1) == pytest.approx(1.0 + L * 4.0)
    # first call, copy-bound: all copies in a row, then the last layer's compute
    assert sp.simulate_call_ms(L, 2, 1, (7.0, 1.0, 0, 0), calls=1) == pytest.approx(L * 7.0 + 1.0)
    # fully resident: after the first call nothing is copied
    assert sp.simulate_call_ms(L, L, 1, (7.0, 1.0, 0, 0), calls=2) == pytest.approx(L * 1.0)
    # one slot: copy and compute strictly alternate
    assert sp.simulate_call_ms(L, 1, 1, (2.0, 3.0, 0, 0), calls=1) == pytest.approx(L * 5.0)
    # copy-bound with R pinned layers: only L - R blobs cross the link per call
    assert sp.simulate_call_ms(L, 4, 1, (7.0, 1.0, 0, 0), wrap=True, calls=3, pinned=2) == pytest.approx((L - 2) * 7.0)


def test_closed_forms_training():
    L, n = 12, 3
    # compute-bound, cheap copies: forward + backward + the last gradient copy; the turn
    # re-uses the resident layers, the first call pays for the first copy
    t = sp.simulate_call_ms(L, n, 1, (0.5, 2.0, 5.0, 1.0), training=True, calls=1)
    assert t == pytest.approx(0.5 + L * 2.0 + L * 5.0 + 1.0)
    # gradient-stream bound: 4 slots ahead at most, then one backward per gradient copy
    t = sp.simulate_call_ms(L, L, 1, (0.0, 1.0, 1.0, 10.0), training=True, calls=2)
    assert t == pytest.approx(L * 1.0 + 1.0 + L * 10.0)


def test_model_argument_errors():
    assert sp.simulate_call_ms(4, 5, 1, (1, 1, 1, 1)) < 0
    assert sp.simulate_call_ms(4, 2, 0, (1, 1, 1, 1)) < 0
    assert sp.simulate_call_ms(4, 2, 1, (-1, 1, 1, 1)) < 0
    assert sp.simulate_call_ms(4, 2, 1, (float("nan"), 1, 1, 1)) < 0
    assert sp.sp_simulate_call_ms(4, 2, 0, 1, 0, 0, 1, None) < 0
    assert sp.simulate_call_ms(4, 2, 1, (1, 1, 1, 1), pinned=2) < 0


def _desc_and_sizes(name="llama7b"):
    w = synth.WORKLOADS[name]
    desc = sp.make_desc(w)
    slot = (sp.sp_layer_blob_bytes(C.byref(desc)) + 4095) // 4096 * 4096
    ws = sp.sp_workspace_bytes(C.byref(desc), 0)
    return w, desc, slot, ws


def test_tuner_picks_the_smallest_window_that_saturates_the_link():
    w, desc, slot, ws = _desc_and_sizes()
    budget = ws + 6 * slot
    # copy-bound (the paper's LLM case, Sec. 4.2): two slots already keep the link busy, and
    # the other four hold pinned layers, which saves 4 of 32 copies per call
    k, p, r, ms = sp.autotune(desc, budget, (7.1, 1.1, 0, 0), wrap=True)
    assert (k, p, r) == (1, 1, 4) and ms == pytest.approx((w.n_layers - 4) * 7.1)
    # whatever it returns is a plan that fits
    rc, pl = sp.plan(desc, k, p, budget, pinned=r)
    assert rc == sp.SP_OK and pl.arena_bytes_used <= budget and pl.n_pinned == r
    # compute-bound: pinning gains nothing, the smallest window wins
    k, p, r, ms = sp.autotune(desc, budget, (1.0, 4.0, 0, 0), wrap=True)
    assert (k, p, r) == (1, 1, 0) and ms == pytest.approx(w.n_layers * 4.0)


def test_tuner_goes_resident_when_the_budget_allows():
    w, desc, slot, ws = _desc_and_sizes()
    k, p, r, ms = sp.autotune(desc, ws + w.n_layers * slot, (7.1, 1.1, 0, 0), wrap=True)
    assert k + p >= w.n_layers and r == 0 and ms == pytest.approx(w.n_layers * 1.1)


def test_tuner_needs_depth_when_copies_are_slower_only_sometimes():
    # compute-bound layer but no wrap-around: the model still returns the smallest window
    # within tolerance, and a tolerance of 0 returns the true optimum
    w, desc, slot, ws = _desc_and_sizes()
    budget = ws + 8 * slot
    cost = (3.0, 4.0, 0, 0)
    k0, p0, r0, best = sp.autotune(desc, budget, cost, wrap=False, tolerance=0.0)
    for kk in range(1, 8):
        for pp in range(1, 8):
            for pin in (0, sp.SP_PIN_AUTO):
                rc, pl = sp.plan(desc, kk, pp, budget, pinned=pin)
                if rc == sp.SP_OK:
                    assert sp.simulate_call_ms(w.n_layers, pl.n_slots, pl.p_eff, cost, calls=3,
                                               pinned=pl.n_pinned) >= best - 1e-9
    k1, p1, r1, ms1 = sp.autotune(desc, budget, cost, wrap=False, tolerance=0.05)
    assert k1 + p1 + r1 <= k0 + p0 + r0 and ms1 <= best * 1.05 + 1e-9


def test_tuner_budget_and_argument_errors():
    w, desc, slot, ws = _desc_and_sizes()
    with pytest.raises(sp.SuperpipeError) as e:
        sp.autotune(desc, ws + slot // 2, (1, 1, 0, 0))
    assert e.value.code == sp.SP_ERR_BUDGET
    with pytest.raises(sp.SuperpipeError):
        sp.autotune(desc, ws + 4 * slot, (1, 1, 0, 0), tolerance=-1.0)
    k, p, r = C.c_int(), C.c_int(), C.c_int()
    assert sp.sp_autotune(None, 1 << 40, 0, 0, None, 0.0, C.byref(k), C.byref(p), C.byref(r), None) == sp.SP_ERR_INVALID_ARG


def test_tuner_over_unit_sizes():
    """Three units per layer are proposed where they pay -- a link-bound stack whose budget then
    holds a whole layer more -- and not on a compute-bound stack (the extra fences cost more than
    nothing is gained), not within the tolerance, and never for training."""
    import ctypes as C

    def budget_of(w, desc, layers):
        blob = (sp.sp_layer_blob_bytes(C.byref(desc)) + 4095) // 4096 * 4096
        return sp.sp_workspace_bytes(C.byref(desc), 0) + layers * blob

    w = synth.WORKLOADS["llama7b"]
    desc = sp.make_desc(w)
    cost = (7.116, 0.95, 0.0, 0.0)                 # measured per-layer copy / forward times, ms
    k1, p1, r1, ms1 = sp.autotune(desc, budget_of(w, desc, 4), cost, wrap=True)
    u, k, p, r, ms = sp.autotune_units(desc, budget_of(w, desc, 4), cost, wrap=True)
    assert (k1, p1, r1) == (1, 1, 2) and (u, k, p, r) == (3, 1, 1, 9)
    # 29 layers' bytes instead of 30, plus 25 us for each of the 57 extra copies
    assert ms == pytest.approx(29 * 7.116 + 57 * 0.025 * 29 / 30, rel=0.01) and ms < ms1 * 0.98
    assert 207.0 < ms < 209.0                      # measured on MI355X: 208.0 ms
    # compute-bound: layer units stay
    v = synth.WORKLOADS["vith"]
    vdesc = sp.make_desc(v)
    u, k, p, r, ms = sp.autotune_units(vdesc, budget_of(v, vdesc, 3), (0.71, 0.973, 0.0, 0.0), wrap=True)
    assert u == 1 and (k, p, r) == sp.autotune(vdesc, budget_of(v, vdesc, 3), (0.71, 0.973, 0.0, 0.0), wrap=True)[:3]
    # training: whole layers
    t = synth.WORKLOADS["train1p3b"]
    tdesc = sp.make_desc(t)
    blob = (sp.sp_layer_blob_bytes(C.byref(tdesc)) + 4095) // 4096 * 4096
    tb = sp.sp_workspace_bytes(C.byref(tdesc), 1) + 3 * blob
    assert sp.autotune_units(tdesc, tb, (1.8, 1.0, 3.5, 3.5), training=1)[0] == 1
