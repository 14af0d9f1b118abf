"""Each HIP kernel against the oracle's op, through the C ABI, element by
element on seeded inputs: sizes span several tiles and a ragged tail."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import stack_oracle as O  # noqa: E402
from paper_2410_08791_amd import binding as sp  # noqa: E402
from tests.gpu_util import (DEV, bf16_vals, dev_f32, dev_u16, host_u16, ptr, rand_bf16,  # noqa: E402
                            stream_ptr)

BF16_EPS = 2.0 ** -8     # half an ulp of bf16, relative


def sync():
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,d", [(37, 256), (5, 4096), (3, 8192), (7, 1280), (1, 64)])
@pytest.mark.parametrize("ln", [False, True])
def test_norm(T, d, ln):
    rng = np.random.default_rng(T * 7 + d + ln)
    h = (rng.standard_normal((T, d)) * 2 + (0.5 if ln else 0)).astype(np.float32)
    gb, g = rand_bf16(rng, d, 0.3)
    g = g + 1.0
    gb = __import__("paper_2410_08791_amd.synth", fromlist=["x"]).f32_to_bf16_bits(g.astype(np.float32))
    g = bf16_vals(gb)
    bb, b = rand_bf16(rng, d, 0.3)
    out = torch.zeros((T, d), dtype=torch.int16, device=DEV)
    hd, gd, bd = dev_f32(h), dev_u16(gb), dev_u16(bb)      # keep the device buffers alive
    rc = sp.spk_norm(stream_ptr(), ptr(hd), ptr(gd), ptr(bd) if ln else None, ptr(out), T, d, 1e-5)
    assert rc == sp.SP_OK
    sync()
    got = bf16_vals(host_u16(out))
    h64 = h.astype(np.float64)
    ref = O.layernorm(h64, g, b, 1e-5) if ln else O.rmsnorm(h64, g, 1e-5)
    assert np.all(np.abs(got - ref) <= BF16_EPS * np.abs(ref) + 1e-5)


def gemm_ref(A, W, epi, R=None, bias=None, N=None):
    acc = A @ W.T
    if bias is not None:
        acc = acc + bias
    if epi == sp.EPI_RESID_F32:
        return R + acc
    if epi == sp.EPI_GELU_BF16:
        return O.gelu(acc)
    if epi == sp.EPI_SWIGLU_BF16:
        return O.silu(acc[:, :N]) * acc[:, N:]
    return acc


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6, 7, 8, 10, 0])
@pytest.mark.parametrize("M,N,K", [(200, 328, 128), (257, 296, 64), (300, 520, 256), (64, 128, 1024)])
@pytest.mark.parametrize("epi", [sp.EPI_BF16, sp.EPI_RESID_F32, sp.EPI_GELU_BF16, sp.EPI_SWIGLU_BF16, sp.EPI_F32])
def test_gemm_kmajor(epi, M, N, K, tile):
    if tile in (8, 10) and epi == sp.EPI_SWIGLU_BF16:
        pytest.skip("the 256x192 and 256x320 tiles do not take the SwiGLU epilogue")
    rng = np.random.default_rng(M + N * 3 + K * 5 + epi)
    Ab, A = rand_bf16(rng, (M, K))
    nw = 2 * N if epi == sp.EPI_SWIGLU_BF16 else N
    Wb, W = rand_bf16(rng, (nw, K), 0.1)
    bias_b, bias = (rand_bf16(rng, N, 0.5) if epi in (sp.EPI_GELU_BF16, sp.EPI_BF16, sp.EPI_RESID_F32) else (None, None))
    R = rng.standard_normal((M, N)).astype(np.float32)
    f32out = epi in (sp.EPI_RESID_F32, sp.EPI_F32)
    Cd = dev_f32(R) if epi == sp.EPI_RESID_F32 else torch.zeros((M, N), dtype=torch.float32 if f32out else torch.int16, device=DEV)
    Ad, Wd = dev_u16(Ab), dev_u16(Wb)
    bd = dev_u16(bias_b) if bias_b is not None else None
    rc = sp.spk_gemm(stream_ptr(), epi, ptr(Ad), K, 0, ptr(Wd), K, 0, ptr(Cd), N,
                     ptr(Cd) if epi == sp.EPI_RESID_F32 else None, N, ptr(bd), M, N, K, tile)
    assert rc == sp.SP_OK
    sync()
    ref = gemm_ref(A, W, epi, R.astype(np.float64), bias, N)
    got = Cd.cpu().numpy().astype(np.float64) if f32out else bf16_vals(host_u16(Cd))
    scale = np.max(np.abs(ref))
    tol = 2e-6 * np.sqrt(K) * scale + (0 if f32out else BF16_EPS * np.abs(ref))
    assert np.all(np.abs(got - ref) <= tol + 1e-6), float(np.max(np.abs(got - ref)))


@pytest.mark.parametrize("tile", [9, 0, 11, 12, 13])
@pytest.mark.parametrize("M,N,K", [(1, 8, 64), (8, 328, 4096), (16, 24, 320), (5, 1288, 1088), (13, 4096, 192),
                                   (17, 40, 448), (32, 328, 1280), (33, 72, 64), (64, 5128, 1280)])
@pytest.mark.parametrize("epi", [sp.EPI_BF16, sp.EPI_RESID_F32, sp.EPI_GELU_BF16, sp.EPI_SWIGLU_BF16, sp.EPI_F32])
def test_gemm_few_rows_streams_the_weights(epi, M, N, K, tile):
    """At most 64 activation rows (a decode step, the ragged last rows of a long launch): the
    weight-streaming kernel, forced (tile 9; 11-13 with 16, 32, 64 rows per work-group, the rest of
    the rows in further work-groups) and as the heuristic's choice; N not a multiple of the
    16 columns of a work-group nor of the 8 column blocks of a dispatch group, K / 32 not a multiple of the eight waves that share the
    contraction, M at and next to the limits of its one, two and four 16-row tiles."""
    rng = np.random.default_rng(M + N * 3 + K * 5 + epi)
    Ab, A = rand_bf16(rng, (M, K))
    nw = 2 * N if epi == sp.EPI_SWIGLU_BF16 else N
    Wb, W = rand_bf16(rng, (nw, K), 0.1)
    bias_b, bias = (rand_bf16(rng, N, 0.5) if epi in (sp.EPI_GELU_BF16, sp.EPI_BF16, sp.EPI_RESID_F32) else (None, None))
    R = rng.standard_normal((M, N)).astype(np.float32)
    f32out = epi in (sp.EPI_RESID_F32, sp.EPI_F32)
    # one guard row behind C: the kernel must not write past row M - 1
    Cd = torch.full((M + 1, N), 7.0 if f32out else 7, dtype=torch.float32 if f32out else torch.int16, device=DEV)
    if epi == sp.EPI_RESID_F32:
        Cd[:M] = dev_f32(R)
    Ad, Wd = dev_u16(Ab), dev_u16(Wb)
    bd = dev_u16(bias_b) if bias_b is not None else None
    rc = sp.spk_gemm(stream_ptr(), epi, ptr(Ad), K, 0, ptr(Wd), K, 0, ptr(Cd), N,
                     ptr(Cd) if epi == sp.EPI_RESID_F32 else None, N, ptr(bd), M, N, K, tile)
    assert rc == sp.SP_OK
    sync()
    ref = gemm_ref(A, W, epi, R.astype(np.float64), bias, N)
    out = Cd.cpu()
    assert bool((out[M] == 7).all())
    got = out[:M].numpy().astype(np.float64) if f32out else bf16_vals(host_u16(out[:M].contiguous()))
    scale = np.max(np.abs(ref))
    tol = 2e-6 * np.sqrt(K) * scale + (0 if f32out else BF16_EPS * np.abs(ref))
    assert np.all(np.abs(got - ref) <= tol + 1e-6), float(np.max(np.abs(got - ref)))


def test_gemm_few_rows_kernel_refuses_what_it_cannot_take():
    z = torch.zeros(1 << 16, dtype=torch.int16, device=DEV)
    f = torch.zeros(1 << 14, dtype=torch.float32, device=DEV)
    # 65 rows; an operand with the row index contiguous
    assert sp.spk_gemm(stream_ptr(), sp.EPI_BF16, ptr(z), 64, 0, ptr(z), 64, 0, ptr(z), 64, None, 0, None, 65, 64, 64, 9) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_gemm(stream_ptr(), sp.EPI_F32, ptr(z), 64, 0, ptr(z), 64, 1, ptr(f), 64, None, 0, None, 8, 64, 64, 9) == sp.SP_ERR_INVALID_ARG
    sync()


def test_gemm_output_rows_not_16_byte_aligned():
    """A bf16 output whose row stride is a multiple of 4 but not of 8 elements: the kernel that
    writes 16-byte pieces of a row cannot take it, the library must fall back by itself (also
    when one of that kernel's tiles is forced) and leave the padding columns alone."""
    M, N, K, ldc = 300, 264, 128, 268
    rng = np.random.default_rng(5)
    Ab, A = rand_bf16(rng, (M, K))
    Wb, W = rand_bf16(rng, (N, K), 0.1)
    Ad, Wd = dev_u16(Ab), dev_u16(Wb)
    ref = A @ W.T
    for tile in (0, 5, 7):
        Cd = torch.full((M, ldc), 0x7fc0, dtype=torch.int16, device=DEV)
        rc = sp.spk_gemm(stream_ptr(), sp.EPI_BF16, ptr(Ad), K, 0, ptr(Wd), K, 0, ptr(Cd), ldc,
                         None, 0, None, M, N, K, tile)
        assert rc == sp.SP_OK
        sync()
        raw = host_u16(Cd)
        got = bf16_vals(raw[:, :N])
        assert np.all(np.abs(got - ref) <= BF16_EPS * np.abs(ref) + 2e-6 * np.sqrt(K) * np.max(np.abs(ref)))
        assert np.all(raw[:, N:] == 0x7fc0)


@pytest.mark.parametrize("epi", [sp.EPI_GELU_BF16, sp.EPI_RESID_F32])
def test_gemm_ragged_rows_cut_off(epi):
    """A shape whose last, ragged row of 256-row tiles would cost a whole extra round: the
    library's own choice computes rows 1024.. in a second launch.  Every row must come out."""
    M, N, K = 1088, 13312, 64
    rng = np.random.default_rng(11 + epi)
    Ab, A = rand_bf16(rng, (M, K))
    Wb, W = rand_bf16(rng, (N, K), 0.1)
    bias_b, bias = rand_bf16(rng, N, 0.5)
    R = rng.standard_normal((M, N)).astype(np.float32)
    f32out = epi == sp.EPI_RESID_F32
    Cd = dev_f32(R) if f32out else torch.zeros((M, N), dtype=torch.int16, device=DEV)
    Ad, Wd, bd = dev_u16(Ab), dev_u16(Wb), dev_u16(bias_b)
    rc = sp.spk_gemm(stream_ptr(), epi, ptr(Ad), K, 0, ptr(Wd), K, 0, ptr(Cd), N,
                     ptr(Cd) if f32out else None, N, ptr(bd), M, N, K, 0)
    assert rc == sp.SP_OK
    sync()
    ref = gemm_ref(A, W, epi, R.astype(np.float64), bias, N)
    got = Cd.cpu().numpy().astype(np.float64) if f32out else bf16_vals(host_u16(Cd))
    tol = 2e-6 * np.sqrt(K) * np.max(np.abs(ref)) + (0 if f32out else BF16_EPS * np.abs(ref))
    assert np.all(np.abs(got - ref) <= tol + 1e-6), float(np.max(np.abs(got - ref)))


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 6, 0])
@pytest.mark.parametrize("M,N,K", [(200, 328, 128), (264, 520, 192)])
def test_gemm_transposed_operands(M, N, K, tile):
    """The backward forms: dX = dY W (weight read with its row index contiguous) and
    dW = dY^T X (both operands transposed on the way in)."""
    rng = np.random.default_rng(M * 3 + N + K + tile)
    Ab, A = rand_bf16(rng, (M, K))
    Wb, W = rand_bf16(rng, (N, K), 0.1)
    # (0,1): W given as [K, N]
    WbT = np.ascontiguousarray(Wb.T)
    C1 = torch.zeros((M, N), dtype=torch.int16, device=DEV)
    Ad, WTd = dev_u16(Ab), dev_u16(WbT)
    rc = sp.spk_gemm(stream_ptr(), sp.EPI_BF16, ptr(Ad), K, 0, ptr(WTd), N, 1, ptr(C1), N,
                     None, 0, None, M, N, K, tile)
    assert rc == sp.SP_OK
    # (1,1): both given transposed, fp32 output
    AbT = np.ascontiguousarray(Ab.T)
    C2 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    ATd = dev_u16(AbT)
    rc = sp.spk_gemm(stream_ptr(), sp.EPI_F32, ptr(ATd), M, 1, ptr(WTd), N, 1, ptr(C2), N,
                     None, 0, None, M, N, K, tile)
    assert rc == sp.SP_OK
    sync()
    ref = A @ W.T
    scale = np.max(np.abs(ref))
    assert np.all(np.abs(bf16_vals(host_u16(C1)) - ref) <= BF16_EPS * np.abs(ref) + 2e-6 * np.sqrt(K) * scale)
    assert np.all(np.abs(C2.cpu().numpy() - ref) <= 2e-6 * np.sqrt(K) * scale)


def test_gemm_rejects_shapes_it_cannot_take():
    z = torch.zeros(1 << 16, dtype=torch.int16, device=DEV)
    args = lambda M, N, K, lda=64, ldw=64, ldc=64: sp.spk_gemm(  # noqa: E731
        stream_ptr(), sp.EPI_BF16, ptr(z), lda, 0, ptr(z), ldw, 0, ptr(z), ldc, None, 0, None, M, N, K, 0)
    assert args(8, 8, 63) == sp.SP_ERR_INVALID_ARG        # K not a multiple of 64
    assert args(8, 7, 64) == sp.SP_ERR_INVALID_ARG        # N not a multiple of 8
    assert args(8, 8, 64, lda=60) == sp.SP_ERR_INVALID_ARG
    assert args(0, 8, 64) == sp.SP_OK                     # empty problem: nothing to do
    assert sp.spk_gemm(stream_ptr(), 9, ptr(z), 64, 0, ptr(z), 64, 0, ptr(z), 64, None, 0, None, 8, 8, 64, 0) == sp.SP_ERR_INVALID_ARG
    sync()


@pytest.mark.parametrize("T,f", [(33, 1024), (7, 11008), (1, 8)])
def test_swiglu(T, f):
    rng = np.random.default_rng(T + f)
    gb, g = rand_bf16(rng, (T, 2 * f), 2.0)
    z = torch.zeros((T, f), dtype=torch.int16, device=DEV)
    gd = dev_u16(gb)
    assert sp.spk_swiglu(stream_ptr(), ptr(gd), ptr(z), T, f) == sp.SP_OK
    sync()
    ref = O.silu(g[:, :f]) * g[:, f:]
    assert np.all(np.abs(bf16_vals(host_u16(z)) - ref) <= BF16_EPS * np.abs(ref) + 1e-6)


@pytest.mark.parametrize("B,S,Hq,Hkv,hd,causal", [
    (2, 128, 4, 4, 64, 1),      # the tiny workload's shape
    (3, 257, 4, 4, 80, 0),      # ViT-like: ragged S, head_dim 80, bidirectional
    (1, 300, 8, 2, 128, 1),     # grouped-query heads, ragged S
    (2, 64, 2, 1, 128, 0),
    (1, 1, 2, 2, 64, 1),        # a single token attends to itself
    (1, 129, 2, 2, 64, 1),      # one query past a block boundary
    (2, 33, 2, 2, 80, 1),       # head_dim 80 (padded 192-byte LDS rows), causal, less than one key tile
    (1, 1, 2, 1, 128, 0),
    (11, 520, 16, 4, 128, 1),   # enough work-groups for the paired causal blocks; ragged last key tile
    # head_dim 80 around the query-block (96 / 128) and key-tile (64) boundaries: three-wave and
    # four-wave work-groups, a last key tile of 1, 32, 33, 63 and 64 keys
    (2, 127, 2, 2, 80, 0), (1, 128, 2, 2, 80, 0), (2, 129, 2, 2, 80, 0), (1, 160, 2, 2, 80, 0), (1, 161, 2, 2, 80, 0),
    (2, 256, 2, 2, 80, 0), (2, 257, 16, 16, 80, 0), (1, 258, 2, 2, 80, 0), (1, 289, 4, 2, 80, 1), (1, 257, 2, 1, 80, 1),
    (1, 96, 2, 2, 80, 1), (1, 97, 2, 2, 80, 0),
    # three-wave work-groups at the other head dims (S = 77: 3 blocks of 32; S = 520: 6 x 96 < 5 x 128)
    (2, 77, 2, 2, 128, 1), (1, 520, 4, 2, 64, 1), (2, 33, 2, 2, 64, 0), (1, 289, 2, 2, 64, 0),
])
def test_attention(B, S, Hq, Hkv, hd, causal):
    rng = np.random.default_rng(B + S + Hq + hd + causal)
    nqkv = (Hq + 2 * Hkv) * hd
    qb, qkv = rand_bf16(rng, (B * S, nqkv))
    sh = O.StackShape(O.DECODER, 1, Hq * hd, Hq, Hkv, hd, 64, bool(causal))
    nq, nk = Hq * hd, Hkv * hd
    q, k, v = qkv[:, :nq], qkv[:, nq:nq + nk], qkv[:, nq + nk:]
    ref = O.attention(q, k, v, B, S, sh)
    o = torch.zeros((B * S, nq), dtype=torch.int16, device=DEV)
    lse = torch.zeros((B, Hq, S), dtype=torch.float32, device=DEV)
    qd = dev_u16(qb)
    rc = sp.spk_attention(stream_ptr(), ptr(qd), ptr(o), ptr(lse), B, S, Hq, Hkv, hd, causal)
    assert rc == sp.SP_OK
    sync()
    got = bf16_vals(host_u16(o))
    # probabilities and the output are each rounded to bf16 once
    assert np.max(np.abs(got - ref)) <= 3 * BF16_EPS * np.max(np.abs(ref))
    # log-sum-exp of the scaled, masked scores
    want = np.empty((B, Hq, S))
    for b in range(B):
        qb_ = q[b * S:(b + 1) * S].reshape(S, Hq, hd)
        kb_ = np.repeat(k[b * S:(b + 1) * S].reshape(S, Hkv, hd), Hq // Hkv, axis=1)
        s = np.einsum("ihd,jhd->hij", qb_, kb_) / np.sqrt(hd)
        if causal:
            s = np.where(np.arange(S)[None, :] <= np.arange(S)[:, None], s, -np.inf)
        m = s.max(-1)
        want[b] = m + np.log(np.exp(s - m[..., None]).sum(-1))
    # head_dim 80: the kernel takes the softmax denominator from the matrix pipe as the sum of the
    # bf16-ROUNDED probabilities (positive terms, each within 2^-9 of its value), so log(sum) is
    # within 2^-9 of the exact one; the other head dims add the fp32 probabilities
    atol = 2e-4 + (2.0 ** -9 if hd == 80 else 0.0)
    np.testing.assert_allclose(lse.cpu().numpy(), want, rtol=0, atol=atol * max(1.0, np.abs(want).max()))


def test_attention_rejects_unsupported_head_dim():
    z = torch.zeros(1 << 16, dtype=torch.int16, device=DEV)
    assert sp.spk_attention(stream_ptr(), ptr(z), ptr(z), None, 1, 8, 2, 2, 48, 1) == sp.SP_ERR_INVALID_ARG
    assert sp.spk_attention(stream_ptr(), ptr(z), ptr(z), None, 1, 8, 3, 2, 64, 1) == sp.SP_ERR_INVALID_ARG
    sync()


# ------------------------------------------------------------------ backward kernels
def test_mse_loss_and_gradient():
    rng = np.random.default_rng(3)
    n = 3 * 77 * 256
    y = rng.standard_normal(n).astype(np.float32)
    t = rng.standard_normal(n).astype(np.float32)
    yd, td = dev_f32(y), dev_f32(t)
    dy = torch.zeros(n, dtype=torch.float32, device=DEV)
    dyb = torch.zeros(n, dtype=torch.int16, device=DEV)
    scratch = torch.zeros(1024, dtype=torch.float32, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    assert sp.spk_mse(stream_ptr(), ptr(yd), ptr(td), ptr(dy), ptr(dyb), ptr(scratch), ptr(loss), n) == sp.SP_OK
    sync()
    ref = O.mse_loss(y.astype(np.float64), t.astype(np.float64))
    assert abs(float(loss.item()) - ref) <= 1e-5 * ref
    dref = 2.0 * (y.astype(np.float64) - t) / n
    np.testing.assert_allclose(dy.cpu().numpy(), dref, rtol=1e-5, atol=1e-12)
    assert np.all(np.abs(bf16_vals(host_u16(dyb)) - dref) <= BF16_EPS * np.abs(dref) + 1e-12)


@pytest.mark.parametrize("T,f", [(33, 1024), (5, 5504)])
def test_swiglu_backward(T, f):
    rng = np.random.default_rng(T + f)
    gb, gu = rand_bf16(rng, (T, 2 * f), 2.0)
    db, dz = rand_bf16(rng, (T, f))
    gud, dzd = dev_u16(gb), dev_u16(db)
    assert sp.spk_swiglu_bwd(stream_ptr(), ptr(dzd), ptr(gud), T, f) == sp.SP_OK
    sync()
    dg, du = O._swiglu_bwd(dz, gu[:, :f], gu[:, f:])
    got = bf16_vals(host_u16(gud))
    ref = np.concatenate([dg, du], axis=1)
    assert np.all(np.abs(got - ref) <= BF16_EPS * np.abs(ref) + 1e-6)


@pytest.mark.parametrize("T,d", [(300, 256), (37, 2048), (5, 8192), (700, 512),
                                 # 1024 rows and more of at most 2048 elements: one wave per row
                                 (1501, 2048), (1100, 320), (1024, 64), (2050, 1280)])
def test_rmsnorm_backward(T, d):
    rng = np.random.default_rng(T * 3 + d)
    da = rng.standard_normal((T, d)).astype(np.float32)
    h = (rng.standard_normal((T, d)) * 1.5).astype(np.float32)
    dh0 = rng.standard_normal((T, d)).astype(np.float32)
    gb, g = rand_bf16(rng, d, 0.3)
    dad, hd, gd, dhd = dev_f32(da), dev_f32(h), dev_u16(gb), dev_f32(dh0)
    dhb = torch.zeros((T, d), dtype=torch.int16, device=DEV)
    scratch = torch.zeros(256 * d, dtype=torch.float32, device=DEV)
    dgain = torch.zeros(d, dtype=torch.float32, device=DEV)
    rc = sp.spk_rmsnorm_bwd(stream_ptr(), ptr(dad), ptr(hd), ptr(gd), ptr(dhd), ptr(dhb), ptr(scratch), ptr(dgain),
                            T, d, 1e-5)
    assert rc == sp.SP_OK
    sync()
    dh_ref, dg_ref = O._rmsnorm_bwd(da.astype(np.float64), h.astype(np.float64), g, 1e-5)
    dh_ref = dh_ref + dh0
    got = dhd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - dh_ref)) <= 1e-5 * np.max(np.abs(dh_ref))
    assert np.max(np.abs(dgain.cpu().numpy() - dg_ref)) <= 1e-5 * np.max(np.abs(dg_ref)) * np.sqrt(T)
    assert np.all(np.abs(bf16_vals(host_u16(dhb)) - got) <= BF16_EPS * np.abs(got) + 1e-12)


@pytest.mark.parametrize("B,S,Hq,Hkv,hd,causal", [
    (2, 128, 4, 4, 64, 1),
    (1, 300, 8, 2, 128, 1),     # grouped-query heads, ragged S
    (2, 77, 2, 2, 128, 0),
    (2, 257, 2, 2, 80, 0),
    (1, 33, 4, 1, 64, 1),
])
def test_attention_backward(B, S, Hq, Hkv, hd, causal):
    rng = np.random.default_rng(B * 5 + S + Hq + hd + causal)
    nq, nk = Hq * hd, Hkv * hd
    nqkv = nq + 2 * nk
    qb, qkv = rand_bf16(rng, (B * S, nqkv))
    dob, dO = rand_bf16(rng, (B * S, nq))
    sh = O.StackShape(O.DECODER, 1, nq, Hq, Hkv, hd, 64, bool(causal))
    q, k, v = qkv[:, :nq], qkv[:, nq:nq + nk], qkv[:, nq + nk:]
    dq, dk, dv = O._attention_bwd(dO, np.ascontiguousarray(q), np.ascontiguousarray(k), np.ascontiguousarray(v), B, S, sh)
    qd, dod = dev_u16(qb), dev_u16(dob)
    o = torch.zeros((B * S, nq), dtype=torch.int16, device=DEV)
    lse = torch.zeros((B, Hq, S), dtype=torch.float32, device=DEV)
    assert sp.spk_attention(stream_ptr(), ptr(qd), ptr(o), ptr(lse), B, S, Hq, Hkv, hd, causal) == sp.SP_OK
    scratch = torch.zeros(sp.spk_attention_bwd_scratch_bytes(B, S, Hq, Hkv, hd), dtype=torch.uint8, device=DEV)
    dqkv = torch.zeros((B * S, nqkv), dtype=torch.int16, device=DEV)
    rc = sp.spk_attention_bwd(stream_ptr(), ptr(qd), ptr(o), ptr(dod), ptr(lse), ptr(scratch), ptr(dqkv),
                              B, S, Hq, Hkv, hd, causal)
    assert rc == sp.SP_OK
    sync()
    got = bf16_vals(host_u16(dqkv))
    for name, g, r in (("dq", got[:, :nq], dq), ("dk", got[:, nq:nq + nk], dk), ("dv", got[:, nq + nk:], dv)):
        err = np.max(np.abs(g - r)) / np.max(np.abs(r))
        assert err <= 1.5e-2, (name, err)


@pytest.mark.parametrize("T,d", [(300, 256), (37, 1280), (5, 8192), (700, 320)])
def test_layernorm_backward(T, d):
    rng = np.random.default_rng(T * 5 + d)
    da = rng.standard_normal((T, d)).astype(np.float32)
    h = (rng.standard_normal((T, d)) * 1.5 + 0.7).astype(np.float32)
    dh0 = rng.standard_normal((T, d)).astype(np.float32)
    gb, g = rand_bf16(rng, d, 0.3)
    dad, hd, gd, dhd = dev_f32(da), dev_f32(h), dev_u16(gb), dev_f32(dh0)
    dhb = torch.zeros((T, d), dtype=torch.int16, device=DEV)
    scratch = torch.zeros(256 * 2 * d, dtype=torch.float32, device=DEV)
    dgain = torch.zeros(d, dtype=torch.float32, device=DEV)
    dbias = torch.zeros(d, dtype=torch.float32, device=DEV)
    rc = sp.spk_layernorm_bwd(stream_ptr(), ptr(dad), ptr(hd), ptr(gd), ptr(dhd), ptr(dhb), ptr(scratch), ptr(dgain),
                              ptr(dbias), T, d, 1e-5)
    assert rc == sp.SP_OK
    sync()
    dh_ref, dg_ref, db_ref = O._layernorm_bwd(da.astype(np.float64), h.astype(np.float64), g, 1e-5)
    dh_ref = dh_ref + dh0
    got = dhd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - dh_ref)) <= 1e-5 * np.max(np.abs(dh_ref))
    assert np.max(np.abs(dgain.cpu().numpy() - dg_ref)) <= 1e-5 * np.max(np.abs(dg_ref)) * np.sqrt(T)
    assert np.max(np.abs(dbias.cpu().numpy() - db_ref)) <= 1e-5 * np.max(np.abs(db_ref)) * np.sqrt(T)
    assert np.all(np.abs(bf16_vals(host_u16(dhb)) - got) <= BF16_EPS * np.abs(got) + 1e-12)


@pytest.mark.parametrize("n", [8, 4096 * 33, 5120 * 7])
def test_gelu_and_its_backward(n):
    rng = np.random.default_rng(n)
    ub, u = rand_bf16(rng, n, 2.0)
    dzb, dz = rand_bf16(rng, n)
    ud, dzd = dev_u16(ub), dev_u16(dzb)
    z = torch.zeros(n, dtype=torch.int16, device=DEV)
    assert sp.spk_gelu(stream_ptr(), ptr(ud), ptr(z), n) == sp.SP_OK
    assert sp.spk_gelu_bwd(stream_ptr(), ptr(dzd), ptr(ud), n) == sp.SP_OK
    sync()
    zr = O.gelu(u)
    assert np.all(np.abs(bf16_vals(host_u16(z)) - zr) <= BF16_EPS * np.abs(zr) + 2e-7)
    # the derivative by central differences of the oracle's gelu in fp64
    e = 1e-6
    dref = dz * (O.gelu(u + e) - O.gelu(u - e)) / (2 * e)
    got = bf16_vals(host_u16(ud))
    assert np.all(np.abs(got - dref) <= BF16_EPS * np.abs(dref) + 1e-6 * np.abs(dz) + 1e-9)
    assert sp.spk_gelu(stream_ptr(), ptr(ud), ptr(z), 12) == sp.SP_ERR_INVALID_ARG


@pytest.mark.parametrize("T,n,ld", [(300, 256, 256), (1000, 3840, 3840), (37, 1280, 2560), (5, 2, 8)])
def test_column_sums(T, n, ld):
    rng = np.random.default_rng(T + n)
    sb, s = rand_bf16(rng, (T, ld))
    sd = dev_u16(sb)
    scratch = torch.zeros(256 * n, dtype=torch.float32, device=DEV)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    assert sp.spk_colsum_bf16(stream_ptr(), ptr(sd), ld, T, n, ptr(scratch), ptr(out)) == sp.SP_OK
    sync()
    ref = s[:, :n].sum(axis=0)
    assert np.max(np.abs(out.cpu().numpy() - ref)) <= 1e-5 * np.sqrt(T) * max(np.max(np.abs(ref)), 1.0)
    assert sp.spk_colsum_bf16(stream_ptr(), ptr(sd), ld, T, 3, ptr(scratch), ptr(out)) == sp.SP_ERR_INVALID_ARG
