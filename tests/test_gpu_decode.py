"""Autoregressive decode against a key/value cache, on the GPU through the C ABI.

What decode computes has a plain definition: with a causal mask, position t of the full
forward over a sequence depends on positions <= t only, so the output of a decode step at
position t must equal row t of the oracle's causal forward over the whole sequence.  The
oracle is used as it stands (no decode-specific code in it)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import stack_oracle as O  # noqa: E402
from paper_2410_08791_amd import binding as sp  # noqa: E402
from paper_2410_08791_amd import synth  # noqa: E402
from tests.gpu_util import DEV, dev_f32, dev_u16, host_u16, bf16_vals, max_rel, ptr, rand_bf16, stack_errs, stream_ptr  # noqa: E402

TOL = 2e-2


def both(got, ref, x):
    """Error against max |ref| and against what the stack added to its input; both <= TOL."""
    d = ref.shape[-1]
    e = stack_errs(got.reshape(-1, d), ref.reshape(-1, d), x.reshape(-1, d))
    return max(e["out"], e["contrib"])


@pytest.mark.parametrize("B,n,max_len,Hq,Hkv,hd", [
    (2, 1, 8, 4, 4, 64), (3, 77, 128, 4, 2, 64), (2, 600, 1024, 8, 2, 128), (1, 1024, 1024, 2, 1, 128),
    (1, 4099, 4104, 2, 2, 64),
])
def test_append_and_single_query_attention(B, n, max_len, Hq, Hkv, hd):
    """Cache n positions with spk_kv_append (in two chunks), then attend the last position's
    query: equals the last row of the oracle's causal attention over the n positions."""
    rng = np.random.default_rng(n * 7 + Hq)
    ld = (Hq + 2 * Hkv) * hd
    bits, vals = rand_bf16(rng, (B, n, ld))
    shape = O.StackShape("decoder", 1, Hq * hd, Hq, Hkv, hd, 64, True, 1e-5)
    q = vals[:, :, :Hq * hd].reshape(B * n, Hq * hd)
    k = vals[:, :, Hq * hd:(Hq + Hkv) * hd].reshape(B * n, Hkv * hd)
    v = vals[:, :, (Hq + Hkv) * hd:].reshape(B * n, Hkv * hd)
    ref = O.attention(q, k, v, B, n, shape).reshape(B, n, Hq * hd)[:, -1]

    kt = torch.zeros(B * Hkv * hd * max_len, dtype=torch.int16, device=DEV)
    vc = torch.zeros(B * Hkv * max_len * hd, dtype=torch.int16, device=DEV)
    cut = n // 3
    for lo, hi in [(0, cut), (cut, n)]:
        if hi > lo:
            chunk = dev_u16(np.ascontiguousarray(bits[:, lo:hi]).reshape(-1))
            assert sp.spk_kv_append(stream_ptr(), ptr(chunk), ptr(kt), ptr(vc), B, hi - lo, lo, Hq, Hkv, hd,
                                    max_len) == sp.SP_OK
    # cache contents, bit for bit
    kt_h = host_u16(kt).reshape(B, Hkv, hd, max_len)[..., :n]
    vc_h = host_u16(vc).reshape(B, Hkv, max_len, hd)[:, :, :n]
    kb = bits[:, :, Hq * hd:(Hq + Hkv) * hd].reshape(B, n, Hkv, hd)
    vb = bits[:, :, (Hq + Hkv) * hd:].reshape(B, n, Hkv, hd)
    assert np.array_equal(kt_h, kb.transpose(0, 2, 3, 1)) and np.array_equal(vc_h, vb.transpose(0, 2, 1, 3))

    last = dev_u16(np.ascontiguousarray(bits[:, -1]).reshape(-1))
    o = torch.zeros(B * Hq * hd, dtype=torch.int16, device=DEV)
    assert sp.spk_decode_attention(stream_ptr(), ptr(last), ptr(kt), ptr(vc), ptr(o), B, n, max_len, Hq, Hkv,
                                   hd) == sp.SP_OK
    torch.cuda.synchronize()
    got = bf16_vals(host_u16(o)).reshape(B, Hq * hd)
    err = max_rel(got, ref)
    print(f"decode attention B={B} n={n} Hq/Hkv={Hq}/{Hkv} hd={hd}: max rel err {err:.3e}")
    assert err <= 8e-3          # one bf16 rounding of the output


def test_decode_kernel_argument_errors():
    t = torch.zeros(1 << 16, dtype=torch.int16, device=DEV)
    s = stream_ptr()
    assert sp.spk_decode_attention(s, ptr(t), ptr(t), ptr(t), ptr(t), 1, 4, 8, 4, 4, 80) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_decode_attention(s, ptr(t), ptr(t), ptr(t), ptr(t), 1, 9, 8, 4, 4, 64) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_decode_attention(s, ptr(t), ptr(t), ptr(t), ptr(t), 1, 4, 7, 4, 4, 64) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_decode_attention(s, ptr(t), ptr(t), ptr(t), ptr(t), 1, 4, 8, 4, 3, 64) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_kv_append(s, ptr(t), ptr(t), ptr(t), 1, 4, 6, 4, 4, 64, 8) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_kv_append(s, None, ptr(t), ptr(t), 1, 4, 0, 4, 4, 64, 8) == sp.SP_ERR_INVALID_ARG
    torch.cuda.synchronize()


class Gen:
    """A small causal decoder stack, its oracle output over S positions, and a runner that
    prefills S0 positions and decodes the rest one by one."""

    def __init__(self, w):
        self.w = w
        self.desc = sp.make_desc(w)
        self.blobs, self.views = sp.pinned_blobs(w, self.desc)
        self.x = synth.make_input(w)                                   # [B, S, d]
        sh = O.StackShape(w.arch, w.n_layers, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn,
                          w.causal, w.norm_eps)
        self.ref = O.stack_forward(self.x, self.views, w.batch, w.seq, sh, dtype=np.float64).reshape(
            w.batch, w.seq, w.d_model)

    def run(self, k, p, s0, max_len, flags=0, pinned=0, budget_layers=None):
        w = self.w
        B, S, d = w.batch, w.seq, w.d_model
        eng = sp.Engine(self.desc, self.blobs, k, p, flags=flags, pinned=pinned, budget_layers=budget_layers)
        cache = torch.empty(sp.sp_kv_cache_bytes(C.byref(self.desc), B, max_len), dtype=torch.uint8, device=DEV)
        cache.fill_(0xFF)                                              # NaN patterns: stale reads would show
        out = np.full((B, S, d), np.nan, dtype=np.float32)
        if s0:
            xd = dev_f32(np.ascontiguousarray(self.x[:, :s0]))
            yd = torch.empty_like(xd)
            eng.prefill(xd, yd, cache, B, s0, max_len)
            eng.sync()
            out[:, :s0] = yd.cpu().numpy()
        for t in range(s0, S):
            xd = dev_f32(np.ascontiguousarray(self.x[:, t]))
            yd = torch.empty_like(xd)
            eng.decode(xd, yd, cache, B, t, max_len)
            eng.sync()
            out[:, t] = yd.cpu().numpy()
        st = eng.stats()
        assert eng.destroy() == sp.SP_OK
        return out, st


@pytest.fixture(scope="module")
def gen():
    # grouped-query heads, 5 layers, 2 sequences of 40 positions
    return Gen(synth.Workload("gen_small", "decoder", 5, 256, 4, 2, 64, 512, True, 2, 40))


def test_decode_matches_the_causal_forward_of_the_oracle(gen):
    out, st = gen.run(1, 1, s0=24, max_len=48)
    assert np.all(np.isfinite(out))
    err_prefill = both(out[:, :24], gen.ref[:, :24], gen.x[:, :24])
    err_decode = both(out[:, 24:], gen.ref[:, 24:], gen.x[:, 24:])
    print(f"gen_small: prefill 24 positions max rel err {err_prefill:.3e}; 16 decode steps {err_decode:.3e}")
    assert err_prefill <= TOL and err_decode <= TOL
    # every decode step streams the whole stack once: 5 copies per call with 2 slots
    assert st.calls == 1 + 16 and st.last_h2d_copies == 5


def test_decode_from_an_empty_cache_and_bits_across_windows(gen):
    base, _ = gen.run(8, 8, s0=0, max_len=40)                          # resident, no prefill
    assert both(base, gen.ref, gen.x) <= TOL
    for k, p, pinned, flags in [(1, 1, 0, 0), (2, 1, 0, sp.SP_FLAG_WRAP_PREFETCH), (1, 1, 2, sp.SP_FLAG_POISON),
                                (1, 2, 0, sp.SP_FLAG_NO_OVERLAP)]:
        out, st = gen.run(k, p, s0=0, max_len=40, flags=flags, pinned=pinned)
        assert np.array_equal(out.view(np.uint32), base.view(np.uint32)), (k, p, pinned, flags)
        assert not st.plan.fully_resident


def test_decode_head_dim_128_and_prefill_equals_forward():
    w = synth.Workload("gen_hd128", "decoder", 2, 512, 4, 4, 128, 1024, True, 3, 21)
    g = Gen(w)
    out, _ = g.run(1, 1, s0=20, max_len=24)
    assert both(out, g.ref, g.x) <= TOL
    # prefill runs the same kernels as sp_forward: same bits
    eng = sp.Engine(g.desc, g.blobs, 1, 1)
    xd = dev_f32(g.x)
    yd = torch.empty_like(xd)
    eng.forward(xd, yd, w.batch, w.seq)
    eng.sync()
    cache = torch.empty(sp.sp_kv_cache_bytes(C.byref(g.desc), w.batch, 24), dtype=torch.uint8, device=DEV)
    y2 = torch.empty_like(xd)
    eng.prefill(xd, y2, cache, w.batch, w.seq, 24)
    eng.sync()
    assert torch.equal(yd, y2)
    eng.destroy()


def test_decode_argument_errors(gen):
    w = gen.w
    eng = sp.Engine(gen.desc, gen.blobs, 1, 1)
    x = torch.zeros(w.batch, w.d_model, device=DEV)
    cache = torch.zeros(sp.sp_kv_cache_bytes(C.byref(gen.desc), w.batch, 16), dtype=torch.uint8, device=DEV)
    for pos, max_len in [(16, 16), (-1, 16), (0, 12), (0, 1 << 20)]:
        with pytest.raises(sp.SuperpipeError) as ex:
            eng.decode(x, x, cache, w.batch, pos, max_len)
        assert ex.value.code == sp.SP_ERR_SHAPE
    with pytest.raises(sp.SuperpipeError):
        eng.prefill(torch.zeros(w.batch, 17, w.d_model, device=DEV), torch.zeros(w.batch, 17, w.d_model, device=DEV),
                    cache, w.batch, 17, 16)
    eng.destroy()
    assert sp.sp_kv_cache_bytes(C.byref(gen.desc), w.batch, 12) == 0
    assert sp.sp_kv_cache_bytes(C.byref(gen.desc), w.batch, 16) == 5 * 2 * w.batch * 2 * 64 * 16 * 2
    # encoder stacks have no causal mask: no cache
    we = synth.WORKLOADS["vith"].with_(n_layers=1, batch=1)
    de = sp.make_desc(we)
    be, _ = sp.pinned_blobs(we, de)
    ee = sp.Engine(de, be, 1, 1)
    xe = torch.zeros(1, we.d_model, device=DEV)
    with pytest.raises(sp.SuperpipeError) as ex:
        ee.decode(xe, xe, cache, 1, 0, 16)
    assert ex.value.code == sp.SP_ERR_STATE
    ee.destroy()
