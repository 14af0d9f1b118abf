"""The entry point that allocates nothing (spk_rmsnorm_bwd_static: partial rows in an array built
into the library) against the entry point it is a variant of (spk_rmsnorm_bwd, caller's scratch
buffer): same kernels, so the results must agree bit for bit; two calls in a row, the second
with a smaller input, so that what the first call left in the shared array must not matter."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import stack_oracle as O  # noqa: E402
from paper_2410_08791_amd import binding as sp  # noqa: E402
from tests.gpu_util import DEV, bf16_vals, dev_f32, dev_u16, host_u16, ptr, rand_bf16, stream_ptr  # noqa: E402


def _case(T, d, seed):
    rng = np.random.default_rng(seed)
    da = rng.standard_normal((T, d)).astype(np.float32)
    h = (rng.standard_normal((T, d)) * 1.5).astype(np.float32)
    dh0 = rng.standard_normal((T, d)).astype(np.float32)
    gb, g = rand_bf16(rng, d, 0.3)
    return da, h, dh0, gb, g


def test_static_scratch_variant_matches_the_caller_scratch_entry_point():
    assert sp.spk_rmsnorm_bwd_static_max_d() == 4096
    for T, d, seed in ((700, 4096, 1), (37, 512, 2)):         # the second call is the smaller one
        da, h, dh0, gb, g = _case(T, d, seed)
        dad, hd, gd = dev_f32(da), dev_f32(h), dev_u16(gb)
        outs = []
        for static in (False, True):
            dhd = dev_f32(dh0)
            dhb = torch.zeros((T, d), dtype=torch.int16, device=DEV)
            dgain = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV)
            if static:
                print(f"spk_rmsnorm_bwd_static T={T} d={d}", flush=True)
                rc = sp.spk_rmsnorm_bwd_static(stream_ptr(), ptr(dad), ptr(hd), ptr(gd), ptr(dhd), ptr(dhb),
                                               ptr(dgain), T, d, 1e-5)
            else:
                scratch = torch.zeros(256 * d, dtype=torch.float32, device=DEV)
                rc = sp.spk_rmsnorm_bwd(stream_ptr(), ptr(dad), ptr(hd), ptr(gd), ptr(dhd), ptr(dhb), ptr(scratch),
                                        ptr(dgain), T, d, 1e-5)
            assert rc == sp.SP_OK
            torch.cuda.synchronize()
            outs.append((dhd.cpu().numpy(), host_u16(dhb).copy(), dgain.cpu().numpy()))
        for a, b in zip(*outs):
            assert np.array_equal(a, b)
        # and against the oracle, to the bar of the caller-scratch entry point's own test
        dh_ref, dg_ref = O._rmsnorm_bwd(da.astype(np.float64), h.astype(np.float64), g, 1e-5)
        dh_ref = dh_ref + dh0
        got = outs[1][0].astype(np.float64)
        assert np.max(np.abs(got - dh_ref)) <= 1e-5 * np.max(np.abs(dh_ref))
        assert np.max(np.abs(outs[1][2] - dg_ref)) <= 1e-5 * np.max(np.abs(dg_ref)) * np.sqrt(T)
        assert np.all(np.abs(bf16_vals(outs[1][1]) - got) <= 2.0 ** -8 * np.abs(got) + 1e-12)


def test_static_scratch_variant_rejects_rows_wider_than_its_array():
    T, d = 4, 8192                                            # fine for spk_rmsnorm_bwd, too wide here
    z = torch.zeros((T, d), dtype=torch.float32, device=DEV)
    zb = torch.zeros((T, d), dtype=torch.int16, device=DEV)
    g = torch.zeros(d, dtype=torch.int16, device=DEV)
    dg = torch.zeros(d, dtype=torch.float32, device=DEV)
    rc = sp.spk_rmsnorm_bwd_static(stream_ptr(), ptr(z), ptr(z), ptr(g), ptr(z), ptr(zb), ptr(dg), T, d, 1e-5)
    assert rc == sp.SP_ERR_SHAPE
    rc = sp.spk_rmsnorm_bwd_static(stream_ptr(), ptr(z), ptr(z), ptr(g), ptr(z), ptr(zb), ptr(dg), T, 6, 1e-5)
    assert rc == sp.SP_ERR_SHAPE
    rc = sp.spk_rmsnorm_bwd_static(stream_ptr(), None, ptr(z), ptr(g), ptr(z), ptr(zb), ptr(dg), T, 64, 1e-5)
    assert rc == sp.SP_ERR_INVALID_ARG
