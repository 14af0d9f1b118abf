"""Seeded random stack configurations against the oracle (float64), through the C ABI.

The hand-picked cases of the other files sit on the workloads' shapes; this one draws layer
kinds, widths, head layouts, head dimensions, depths, ragged token counts and window settings
from a seeded generator, within what sp_create accepts, so that the combinations nobody thought
of are met too: every configuration must match the oracle within the task's bound (on the
output and on what the stack adds to its input), and its streamed run must be bit for bit the
resident one (the paper's invariant, Sec. 4.2); the training configurations also check loss, dx
and every weight gradient."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2410_08791_amd import synth  # noqa: E402
from tests.test_gpu_stack import Case, check  # noqa: E402
from tests.test_gpu_train import TrainCase, check_against_oracle  # noqa: E402

N_FORWARD, N_TRAIN = 16, 8


def draw(seed, training):
    """One configuration that sp_create accepts (d_model, d_ffn and the fused q/k/v width multiples
    of 64; head_dim 64, 80 or 128; n_kv_heads divides n_q_heads)."""
    rng = np.random.default_rng([20241008, seed, int(training)])
    arch = "decoder" if rng.random() < 0.6 else "encoder"
    hd = int(rng.choice([64, 80, 128]))
    while True:
        n_kv = int(rng.choice([1, 2, 4]))
        grp = int(rng.choice([1, 2, 4])) if arch == "decoder" else 1
        n_q = n_kv * grp
        if (n_q * hd) % 64 == 0 and ((n_q + 2 * n_kv) * hd) % 64 == 0 and n_q * hd <= 1024:
            break
    d_model = 64 * int(rng.integers(1, 9))
    d_ffn = 64 * int(rng.integers(1, 25))
    n_layers = int(rng.integers(1, 6))
    batch = int(rng.integers(1, 5))
    # ragged lengths on purpose: 1, just around the 32/64/128-row tiles, and anything up to 300
    seq = int(rng.choice([1, 2, 31, 33, 63, 65, 127, 129, int(rng.integers(3, 301))]))
    causal = bool(arch == "decoder" and rng.random() < 0.7)
    k, p = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    w = synth.Workload(f"rand{'_t' if training else ''}{seed}", arch, n_layers, d_model, n_q, n_kv, hd, d_ffn, causal,
                       batch, seq, k=k, p=p, training=training, seed=1000 + seed)
    units = 3 if (not training and rng.random() < 0.3) else 1
    return w, units


def describe(w, units):
    return (f"{w.name}: {w.arch} L={w.n_layers} d={w.d_model} heads={w.n_q_heads}/{w.n_kv_heads}x{w.head_dim} "
            f"ffn={w.d_ffn} causal={w.causal} batch {w.batch} x seq {w.seq}, window ({w.k},{w.p}), units/layer {units}")


@pytest.mark.parametrize("seed", range(N_FORWARD))
def test_random_forward_configuration(seed):
    w, units = draw(seed, False)
    print(describe(w, units), flush=True)
    c = Case(w)
    (y,), st = c.run(w.k, w.p, units=units)
    assert np.all(np.isfinite(y))
    check(y, c.ref(), c.x, w.name)
    (res,), st_res = c.run(w.n_layers, w.n_layers)
    assert st_res.plan.fully_resident
    assert np.array_equal(y.view(np.uint32), res.view(np.uint32)), "streamed and resident runs differ"


@pytest.mark.parametrize("seed", range(N_TRAIN))
def test_random_training_configuration(seed):
    w, _ = draw(seed, True)
    print(describe(w, 1), flush=True)
    c = TrainCase(w)
    got = c.run(w.k, w.p)
    check_against_oracle(got, c.oracle(), w.name)
    res = c.run(w.n_layers, w.n_layers)
    assert got["loss"] == res["loss"]
    assert np.array_equal(got["dx"], res["dx"]) and np.array_equal(got["y"], res["y"])
    for gl, rl in zip(got["grads"], res["grads"]):
        for n in gl:
            assert np.array_equal(gl[n], rl[n]), n
