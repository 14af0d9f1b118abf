"""The C-ABI library loads on a CPU-only box, exports every symbol the headers
declare, and its host-only entry points (layout, plan, schedule trace, argument
checks) behave as documented.  No compute calls here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2410_08791_amd import binding as sp
from paper_2410_08791_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(spk?_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"sp_create", "sp_forward", "sp_forward_backward", "sp_destroy"} <= names
    for n in names:
        assert hasattr(sp.lib, n), f"{n} declared in include/ but not exported"
    assert names == set(sp.EXPORTS), names ^ set(sp.EXPORTS)


@pytest.mark.parametrize("name,blob_bytes", [("tiny", 2098176), ("llama7b", 404766720),
                                             ("vith", 39354880), ("llama70b", 1711308800),
                                             ("train1p3b", 101195776)])
def test_blob_layout(name, blob_bytes):
    w = synth.WORKLOADS[name]
    d = sp.make_desc(w)
    assert sp.sp_layer_blob_bytes(C.byref(d)) == blob_bytes
    assert sp.sp_layer_grad_bytes(C.byref(d)) == 2 * blob_bytes
    specs = synth.tensor_specs(w)
    assert sp.sp_num_tensors(C.byref(d)) == len(specs)
    assert [n for n, _, _ in specs] == sp.TENSOR_NAMES[d.arch]
    prev_end = 0
    for i, (n, shape, _) in enumerate(specs):
        off = sp.sp_tensor_offset(C.byref(d), i)
        cnt = sp.sp_tensor_elems(C.byref(d), i)
        assert cnt == int(np.prod(shape))
        assert off % 256 == 0 and off >= prev_end
        prev_end = off + 2 * cnt
    assert prev_end <= blob_bytes
    assert sp.sp_tensor_offset(C.byref(d), len(specs)) == C.c_size_t(-1).value
    assert sp.sp_tensor_elems(C.byref(d), -1) == 0


def test_blob_views_cover_disjoint_ranges():
    w = synth.WORKLOADS["tiny"]
    d = sp.make_desc(w)
    blob = np.zeros(sp.sp_layer_blob_bytes(C.byref(d)), dtype=np.uint8)
    v = sp.blob_views(d, blob)
    for i, (n, a) in enumerate(v.items()):
        a[:] = i + 1
    for i, (n, a) in enumerate(v.items()):
        assert np.all(a == i + 1), n


def test_bad_descs_are_rejected():
    w = synth.WORKLOADS["tiny"]
    for field, val in [("struct_size", 4), ("n_layers", 0), ("d_model", 100), ("head_dim", 48),
                       ("n_kv_heads", 3), ("d_ffn", 1000), ("arch", 7), ("max_batch", 0), ("norm_eps", 0.0)]:
        d = sp.make_desc(w)
        setattr(d, field, val)
        assert sp.sp_layer_blob_bytes(C.byref(d)) == 0, field
        assert sp.sp_num_tensors(C.byref(d)) == sp.SP_ERR_INVALID_ARG, field
        rc, _ = sp.plan(d, 1, 1, 1 << 40)
        assert rc == sp.SP_ERR_INVALID_ARG, field
    assert sp.sp_layer_blob_bytes(None) == 0
    # head_dim 80 with an odd number of key/value heads: the fused q/k/v width (a contraction
    # length of the backward pass) is not a multiple of 64 -- refused at create, not mid-step
    d = sp.make_desc(synth.WORKLOADS["vith"])
    d.n_q_heads, d.n_kv_heads = 4, 1
    assert sp.sp_layer_blob_bytes(C.byref(d)) == 0
    d.n_kv_heads = 2
    assert sp.sp_layer_blob_bytes(C.byref(d)) > 0


def test_forward_workspace_holds_no_gate_up_buffer():
    """SwiGLU / GELU are applied in the producing GEMM's epilogue: a forward-only handle reserves
    the normed input, q/k/v, the attention output and z, nothing of width 2f."""
    w = synth.WORKLOADS["llama7b"]
    d = sp.make_desc(w)
    T, dm, f = w.tokens, w.d_model, w.d_ffn
    want = 2 * T * (dm + 3 * dm + dm + f)
    got = sp.sp_workspace_bytes(C.byref(d), 0)
    assert want <= got <= want + 5 * 4096
    # and the 4-layer budget of the workload now pins a tenth unit
    blob = sp.sp_layer_blob_bytes(C.byref(d))
    slot = (blob + 4095) // 4096 * 4096
    pl = sp.sp_plan()
    assert sp.sp_make_plan_units(C.byref(d), 3, 1, 1, sp.SP_PIN_AUTO, got + 4 * slot, 0, C.byref(pl)) == sp.SP_OK
    assert pl.arena_bytes_used <= got + 4 * slot


def test_slot_count_policy():
    w = synth.WORKLOADS["llama7b"]
    d = sp.make_desc(w)
    slot = 404766720  # already a multiple of 4096
    ws = sp.sp_workspace_bytes(C.byref(d), 0)
    assert ws > 0 and ws % 4096 == 0
    budget = ws + 4 * slot                      # "HBM budget capped at 4 resident layers"
    got = {}
    for k in (1, 2, 4):
        for p in (1, 2):
            rc, pl = sp.plan(d, k, p, budget)
            assert rc == sp.SP_OK
            got[(k, p)] = (pl.n_slots, pl.k_eff, pl.p_eff)
            assert pl.arena_bytes_used == ws + pl.n_slots * slot <= budget
            assert pl.slot_bytes == slot and pl.workspace_bytes == ws and not pl.fully_resident
    assert got == {(1, 1): (2, 1, 1), (1, 2): (3, 1, 2), (2, 1): (3, 2, 1), (2, 2): (4, 2, 2),
                   (4, 1): (4, 3, 1), (4, 2): (4, 2, 2)}
    # budget below workspace + one slot
    rc, _ = sp.plan(d, 1, 1, ws + slot - 1)
    assert rc == sp.SP_ERR_BUDGET
    # exactly one slot: serialised, p_eff = k_eff = 1
    rc, pl = sp.plan(d, 2, 2, ws + slot)
    assert rc == sp.SP_OK and (pl.n_slots, pl.k_eff, pl.p_eff) == (1, 1, 1)
    # plenty of memory: clamped by the layer count -> fully resident
    rc, pl = sp.plan(d, 40, 2, 1 << 45)
    assert rc == sp.SP_OK and pl.n_slots == 32 and pl.fully_resident
    for k, p in [(0, 1), (1, 0), (-1, 1)]:
        assert sp.plan(d, k, p, budget)[0] == sp.SP_ERR_INVALID_ARG
    # pinned layers take what the budget leaves after the window
    got = {}
    for (k, p, pin) in [(1, 1, sp.SP_PIN_AUTO), (2, 1, sp.SP_PIN_AUTO), (2, 2, sp.SP_PIN_AUTO), (1, 1, 1), (1, 1, 5),
                        (2, 2, 3)]:
        rc, pl = sp.plan(d, k, p, budget, pinned=pin)
        assert rc == sp.SP_OK and pl.arena_bytes_used == ws + pl.n_slots * slot <= budget
        got[(k, p, pin)] = (pl.n_slots, pl.n_pinned, pl.k_eff, pl.p_eff)
    assert got == {(1, 1, -1): (4, 2, 1, 1), (2, 1, -1): (4, 1, 2, 1), (2, 2, -1): (4, 0, 2, 2),
                   (1, 1, 1): (3, 1, 1, 1), (1, 1, 5): (4, 2, 1, 1), (2, 2, 3): (4, 0, 2, 2)}
    rc, pl = sp.plan(d, 2, 2, ws + 40 * slot, pinned=sp.SP_PIN_AUTO)      # everything fits
    assert rc == sp.SP_OK and pl.fully_resident and pl.n_slots == 32 and pl.n_pinned == 0
    rc, pl = sp.plan(d, 2, 2, ws + 31 * slot, pinned=sp.SP_PIN_AUTO)      # one layer short of resident
    assert rc == sp.SP_OK and not pl.fully_resident and (pl.n_slots, pl.n_pinned) == (31, 27)
    assert sp.plan(d, 1, 1, budget, pinned=-2)[0] == sp.SP_ERR_INVALID_ARG
    # training workspace is larger (saved inputs, gradient slots)
    wt = synth.WORKLOADS["train1p3b"]
    dt = sp.make_desc(wt)
    assert sp.sp_workspace_bytes(C.byref(dt), 1) > sp.sp_workspace_bytes(C.byref(dt), 0) + 24 * 8192 * 2048 * 4


def test_create_argument_errors_without_a_device():
    w = synth.WORKLOADS["tiny"]
    d = sp.make_desc(w)
    h = C.c_void_p()
    blob = np.zeros(sp.sp_layer_blob_bytes(C.byref(d)), dtype=np.uint8)
    ptrs = (C.c_void_p * 4)(*[blob.ctypes.data] * 4)
    cfg = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 1 << 30, 4096, None, 8, None, 0)
    assert sp.sp_create(None, C.byref(d), ptrs, C.byref(cfg)) == sp.SP_ERR_INVALID_ARG
    assert sp.sp_create(C.byref(h), None, ptrs, C.byref(cfg)) == sp.SP_ERR_INVALID_ARG
    assert b"desc" in sp.sp_last_error(None)
    assert sp.sp_create(C.byref(h), C.byref(d), None, C.byref(cfg)) == sp.SP_ERR_INVALID_ARG
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, None) == sp.SP_ERR_INVALID_ARG
    bad = sp.sp_config(C.sizeof(sp.sp_config), 0, 1, 1 << 30, 4096, None, 8, None, 0)
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(bad)) == sp.SP_ERR_INVALID_ARG
    bad = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 1 << 30, 4097, None, 8, None, 0)       # misaligned arena
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(bad)) == sp.SP_ERR_INVALID_ARG
    bad = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 1 << 30, 4096, None, None, None, 0)    # same streams
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(bad)) == sp.SP_ERR_INVALID_ARG
    bad = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 1 << 30, 4096, None, 8, None, sp.SP_FLAG_DELAY)
    bad.delay_us = 10 ** 6                                                                  # beyond the bound
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(bad)) == sp.SP_ERR_INVALID_ARG
    bad = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 1 << 30, 4096, None, 8, None, sp.SP_FLAG_TRAINING)
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(bad)) == sp.SP_ERR_INVALID_ARG  # no d2h stream
    small = sp.sp_config(C.sizeof(sp.sp_config), 1, 1, 4096, 4096, None, 8, None, 0)
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(small)) == sp.SP_ERR_BUDGET
    assert b"budget" in sp.sp_last_error(None)
    # pageable numpy memory is not pinned host memory
    assert sp.sp_create(C.byref(h), C.byref(d), ptrs, C.byref(cfg)) == sp.SP_ERR_NOT_PINNED
    assert not h.value
    # calls on a handle that was never created
    assert sp.sp_destroy(None) == sp.SP_ERR_INVALID_ARG
    fake = C.c_void_p(0x1000)
    assert sp.sp_destroy(fake) == sp.SP_ERR_STATE
    assert sp.sp_forward(fake, 16, 16, 1, 1) == sp.SP_ERR_STATE
    assert sp.sp_get_stats(fake, C.byref(sp.sp_stats())) == sp.SP_ERR_STATE


def gemm_plan(epi, a_form, w_form, M, N):
    out = (C.c_int * 3)()
    assert sp.lib.spk_gemm_plan(epi, a_form, w_form, M, N, out) == sp.SP_OK
    return tuple(out)


def test_gemm_plan_is_a_function_of_the_shape_alone():
    """What tile = 0 resolves to: valid ids, the whole of M covered, the SwiGLU epilogue never on
    the tile that cannot pair gate and up rows, the operand forms the LDS-DMA kernel does not take
    on the register-staged tiles, and the workloads' projections on the tiles their round counts
    call for (256 work-groups run at a time)."""
    for epi in range(5):
        for M in (1, 8, 16, 17, 64, 65, 200, 256, 300, 2048, 4096, 8192, 16448):
            for N in (8, 128, 1280, 4096, 5120, 11008, 12288, 28672):
                tile, body, tail_tile = gemm_plan(epi, 0, 0, M, N)
                if M <= 64:           # a decode step: the weight-streaming kernel
                    assert (tile, body, tail_tile) == (9, M, 0)
                    assert gemm_plan(epi, 0, 1, M, N)[0] in (1, 4)
                    continue
                assert tile in (5, 6, 7, 8, 10) and 0 < body <= M
                assert (tail_tile == 0) == (body == M)
                if body < M:
                    assert body % 256 == 0 and M - body < 256 and tail_tile in (5, 6, 7, 8, 9, 10)
                    assert (tail_tile == 9) == (M - body <= 64)
                if epi == sp.EPI_SWIGLU_BF16:
                    assert tile not in (8, 10) and tail_tile not in (8, 10)
                assert gemm_plan(epi, 0, 0, M, N) == (tile, body, tail_tile)
                for forms in ((0, 1), (1, 1), (1, 0)):
                    t, b, tt = gemm_plan(epi, forms[0], forms[1], M, N)
                    assert t in (1, 4) and b == M and tt == 0
    # llama7b, 2048 tokens: gate/up 8 x 86 = 688 tiles of 256x256; QKV 8 x 64 = 512 tiles of 256x192
    # (two full rounds) instead of 384 of 256x256; O and down 16 x 16 = 256 tiles of 128x256 (one round)
    assert gemm_plan(sp.EPI_SWIGLU_BF16, 0, 0, 2048, 11008) == (5, 2048, 0)
    assert gemm_plan(sp.EPI_BF16, 0, 0, 2048, 12288) == (8, 2048, 0)
    assert gemm_plan(sp.EPI_RESID_F32, 0, 0, 2048, 4096) == (6, 2048, 0)
    # ViT-H, 16448 tokens = 64 x 256 + 64: the first MLP projection would take 1300 tiles of 256x256 =
    # 5.08 rounds; cut, it takes 1024 tiles of 256x320 (4 rounds) plus a small launch for the last 64
    # rows; the projections back to d_model = 1280 = 4 x 320 become exactly one round
    assert gemm_plan(sp.EPI_GELU_BF16, 0, 0, 16448, 5120) == (10, 16384, 9)
    assert gemm_plan(sp.EPI_RESID_F32, 0, 0, 16448, 1280) == (10, 16384, 9)
    # llama70b QKV, 4096 x 10240: 512 tiles of 256x320 (two rounds) instead of 640 of 256x256 (2.5)
    assert gemm_plan(sp.EPI_BF16, 0, 0, 4096, 10240) == (10, 4096, 0)
    assert sp.lib.spk_gemm_plan(7, 0, 0, 8, 8, (C.c_int * 3)()) == sp.SP_ERR_INVALID_ARG
    assert sp.lib.spk_gemm_plan(0, 0, 0, 0, 8, (C.c_int * 3)()) == sp.SP_ERR_INVALID_ARG


def test_unit_ranges_and_the_plan_in_units():
    """A layer streamed as three units: the parts tile the blob at tensor boundaries, the plan
    with one unit per layer is sp_make_plan's, and at the llama7b budget of four layers the
    window of two gate/up-sized slots leaves room to pin three whole layers instead of two."""
    w = synth.WORKLOADS["llama7b"]
    desc = sp.make_desc(w)
    blob = sp.sp_layer_blob_bytes(C.byref(desc))
    parts = []
    for q in range(3):
        off, n = C.c_uint64(), C.c_uint64()
        assert sp.sp_unit_range(C.byref(desc), 3, q, C.byref(off), C.byref(n)) == sp.SP_OK
        parts.append((off.value, n.value))
    assert parts[0][0] == 0 and parts[1][0] == sp.sp_tensor_offset(C.byref(desc), 3)   # second norm gain
    assert parts[2][0] == sp.sp_tensor_offset(C.byref(desc), 5)   # down projection
    assert sum(n for _, n in parts) == blob
    off, n = C.c_uint64(), C.c_uint64()
    assert sp.sp_unit_range(C.byref(desc), 1, 0, C.byref(off), C.byref(n)) == sp.SP_OK and (off.value, n.value) == (0, blob)
    assert sp.sp_unit_range(C.byref(desc), 2, 0, C.byref(off), C.byref(n)) == sp.SP_ERR_INVALID_ARG
    assert sp.sp_unit_range(C.byref(desc), 3, 3, C.byref(off), C.byref(n)) == sp.SP_ERR_INVALID_ARG

    ws = sp.sp_workspace_bytes(C.byref(desc), 0)
    al = lambda v: (v + 4095) // 4096 * 4096  # noqa: E731
    budget = ws + 4 * al(blob)
    a, b = sp.sp_plan(), sp.sp_plan()
    for k, p, pinned in [(1, 1, 0), (2, 2, 0), (1, 1, sp.SP_PIN_AUTO), (4, 2, 1), (40, 1, 0)]:
        assert sp.sp_make_plan(C.byref(desc), k, p, pinned, budget, 0, C.byref(a)) == sp.SP_OK
        assert sp.sp_make_plan_units(C.byref(desc), 1, k, p, pinned, budget, 0, C.byref(b)) == sp.SP_OK
        assert bytes(a) == bytes(b) and a.units_per_layer == 1
        assert a.pinned_bytes == a.n_pinned * a.slot_bytes
    # layer units: 2 window slots + 2 pinned layers; three units per layer: 2 slots + 9 pinned units
    assert sp.sp_make_plan(C.byref(desc), 1, 1, sp.SP_PIN_AUTO, budget, 0, C.byref(a)) == sp.SP_OK
    assert (a.n_slots, a.n_pinned) == (4, 2)
    assert sp.sp_make_plan_units(C.byref(desc), 3, 1, 1, sp.SP_PIN_AUTO, budget, 0, C.byref(b)) == sp.SP_OK
    assert b.slot_bytes == al(max(n for _, n in parts)) and (b.n_slots, b.n_pinned) == (11, 9)
    assert b.pinned_bytes == 3 * sum(al(n) for _, n in parts)
    assert b.arena_bytes_used == ws + b.pinned_bytes + 2 * b.slot_bytes <= budget
    assert not b.fully_resident and b.k_eff == 1 and b.p_eff == 1
    # a stack that fits only with the units at their own sizes keeps one unit streaming
    small = sp.make_desc(w, n_layers=2)
    ws2 = sp.sp_workspace_bytes(C.byref(small), 0)
    room = 2 * sum(al(n) for _, n in parts) + al(parts[1][1])
    assert sp.sp_make_plan_units(C.byref(small), 3, 1, 1, sp.SP_PIN_AUTO, ws2 + room, 0, C.byref(b)) == sp.SP_OK
    assert not b.fully_resident and b.n_slots == 5 and b.n_pinned == 3
    assert sp.sp_make_plan_units(C.byref(small), 3, 8, 8, 0, ws2 + 6 * b.slot_bytes, 0, C.byref(b)) == sp.SP_OK
    assert b.fully_resident and b.n_slots == 6 and b.n_pinned == 0 and b.pinned_bytes == 0
    # training handles stream whole layers
    assert sp.sp_make_plan_units(C.byref(desc), 3, 1, 1, 0, 10 * budget, 1, C.byref(b)) == sp.SP_ERR_INVALID_ARG
