"""The seeded generators: bf16 rounding pinned to hand-worked bit patterns,
determinism, and the stated distributions.  CPU only."""
import numpy as np

from paper_2410_08791_amd import synth


def test_bf16_round_to_nearest_even_hand_cases():
    # 1.0 = 0x3F800000.  One bf16 ulp at 1.0 is 2^-7.
    cases = {
        0x3F800000: 0x3F80,   # exact
        0x3F808000: 0x3F80,   # tie -> even (down)
        0x3F818000: 0x3F82,   # tie -> even (up)
        0x3F808001: 0x3F81,   # just above tie -> up
        0x3F807FFF: 0x3F80,   # just below tie -> down
        0xBF808001: 0xBF81,   # sign carried
        0x00000000: 0x0000,
    }
    src = np.array(list(cases.keys()), dtype=np.uint32).view(np.float32)
    assert synth.f32_to_bf16_bits(src).tolist() == list(cases.values())
    back = synth.bf16_bits_to_f32(np.array([0x3F80, 0xC000], dtype=np.uint16))
    assert back.tolist() == [1.0, -2.0]


def test_layers_are_deterministic_and_distinct():
    w = synth.WORKLOADS["tiny"]
    a = synth.make_layer(w, 0)
    b = synth.make_layer(w, 0)
    c = synth.make_layer(w, 1)
    d = synth.make_layer(w, 0, seed=1)
    for n in a:
        assert np.array_equal(a[n], b[n])
        assert not np.array_equal(a[n], c[n])
        assert not np.array_equal(a[n], d[n])
    assert sum(v.size for v in a.values()) == synth.params_per_layer(w) == 1049088


def test_distributions():
    w = synth.WORKLOADS["tiny"]
    a = synth.make_layer(w, 2)
    m = synth.bf16_bits_to_f32(a["wgu"]).astype(np.float64)
    assert abs(m.mean()) < 2e-4 and abs(m.std() - 0.02) < 2e-4
    g = synth.bf16_bits_to_f32(a["g1"]).astype(np.float64)
    assert abs(g.mean() - 1.0) < 0.01 and 0.01 < g.std() < 0.03
    x = synth.make_input(w)
    assert x.shape == (2, 128, 256) and x.dtype == np.float32
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02
    assert not np.array_equal(x, synth.make_input(w, "target"))


def test_param_counts_match_the_named_models():
    assert synth.params_per_layer(synth.WORKLOADS["llama7b"]) == 202383360
    assert synth.params_per_layer(synth.WORKLOADS["vith"]) == 19677440
    assert synth.params_per_layer(synth.WORKLOADS["llama70b"]) == 855654400
    assert synth.params_per_layer(synth.WORKLOADS["train1p3b"]) == 50597888
