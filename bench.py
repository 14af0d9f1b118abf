#!/usr/bin/env python3
"""Headline benchmark: tokens/s of the layer-streamed stack at a fixed HBM
weight budget, on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W            # the headline workload (+ short runs of the others)
    python bench.py --workload vith|llama70b|train1p3b ...   # another workload as the headline

Default workload = the LLaMA-7B-shaped stack (32 layers, d 4096, 32 heads x
128, SwiGLU 11008, causal, batch 1 x seq 2048), bf16 weights in pinned host
memory, HBM weight budget of 4 layer slots; the window -- (k, p), pinned units,
and whether a layer streams whole or as three units -- is chosen at that budget
by the tuner plus a short measured comparison.  A step is one pass of the whole
hot path: sp_forward over the whole stack (every layer that is not held in the
budget copied host-to-device once, every layer computed once), or for the training workload
one sp_forward_backward (forward, loss, backward with re-streamed weights and
gradients streamed device-to-host).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line; `other_workloads` in it holds short timed runs of the
remaining workloads of the list (each with its own roofline and parity sample).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
LINK_NOMINAL_GBPS = 64.0      # PCIe Gen5 x16, one direction


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def overlap_metrics(copy_busy_ms, copy_hidden_ms, compute_busy_ms, wall_ms):
    """Overlap figures of ONE call from its own per-layer trace (sp_stats of a SP_FLAG_TIMING handle).

    copy_hidden_frac       share of the copy time that lay under some layer's compute; when the
                           pass is link-bound it cannot exceed compute/copy (reported as its bound)
    overlap_efficiency     (T_copy + T_compute - T_wall) / min(T_copy, T_compute): 1 = everything
                           that could be hidden was hidden.  All three times belong to the same
                           call; each stream runs its operations one after the other, so
                           T_copy <= T_wall and T_compute <= T_wall and the value lies in [0, 1]
    copy_stream_idle_frac  1 - T_copy / T_wall
    """
    out = {"copy_hidden_frac": None, "copy_hidden_frac_bound": None, "overlap_efficiency": None,
           "copy_stream_idle_frac": None}
    if copy_busy_ms > 0:
        out["copy_hidden_frac"] = round(copy_hidden_ms / copy_busy_ms, 4)
        out["copy_hidden_frac_bound"] = round(min(1.0, compute_busy_ms / copy_busy_ms), 4)
    lo = min(copy_busy_ms, compute_busy_ms)
    if lo > 0 and wall_ms > 0:
        out["overlap_efficiency"] = round((copy_busy_ms + compute_busy_ms - wall_ms) / lo, 4)
    if wall_ms > 0:
        out["copy_stream_idle_frac"] = round(max(0.0, 1.0 - copy_busy_ms / wall_ms), 4)
    return out


def op_work(w, training):
    """Algorithmic work of one step per operation kind of SP_FLAG_OP_TIMING: {name: (bound, amount)},
    amount in FLOP for the contractions (2 M N K; attention 4 B Hq S^2 hd, half when causal, 10 for
    its backward) and in bytes for the HBM-bound kernels (each operand read or written once)."""
    T, L, d, f = w.tokens, w.n_layers, w.d_model, w.d_ffn
    nq, nkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    nqkv = nq + 2 * nkv
    dec = w.arch == "decoder"
    f1 = 2 * f if dec else f
    attn = 4.0 * w.batch * w.n_q_heads * w.seq * w.seq * w.head_dim * (0.5 if w.causal else 1.0)
    mats = d * nqkv + nq * d + d * f1 + f * d                 # matrix elements of a layer
    fwd_passes = 2 if training else 1                         # the backward recomputes the layer
    out = {
        "norm": ("hbm", fwd_passes * L * 2 * T * 6.0 * d),
        "gemm_qkv": ("mfma", fwd_passes * L * 2.0 * T * nqkv * d),
        "attention": ("mfma", fwd_passes * L * attn),
        "gemm_o": ("mfma", fwd_passes * L * 2.0 * T * d * nq),
        "gemm_ffn1": ("mfma", fwd_passes * L * 2.0 * T * d * f1),
        # forward pass only: the recompute stops before the last projection
        "gemm_ffn2": ("mfma", L * 2.0 * T * f * d),
        "copy": ("hbm", 8.0 * T * d * (2 if training else 1)),
    }
    if training:
        out.update({
            "act": ("hbm", fwd_passes * L * T * f * (6.0 if dec else 4.0)),
            "loss": ("hbm", 14.0 * T * d),
            "gemm_dw": ("mfma", L * 2.0 * T * mats),
            "gemm_dx": ("mfma", L * 2.0 * T * mats),
            "act_bwd": ("hbm", L * T * f * (10.0 if dec else 6.0)),
            "norm_bwd": ("hbm", L * 2 * T * 18.0 * d),
            "attention_bwd": ("mfma", L * 2.5 * attn),
            "bias_grad": ("hbm", 0.0 if dec else L * 2.0 * T * (2 * d + nqkv + f)),
        })
    return out


def copy_ceiling_gbps(torch, nbytes=1 << 30, reps=3):
    """Plain pinned hipMemcpyAsync host->device rate, measured in this run."""
    src = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    src.fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    # on the default stream: a stream of its own would be one more than the hardware
    # queues HIP gives a process, and the engine's copy streams would then share one
    st = torch.cuda.current_stream()
    best = 0.0
    dst.copy_(src, non_blocking=True)
    st.synchronize()
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        dst.copy_(src, non_blocking=True)
        e1.record(st)
        st.synchronize()
        best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    return best


def host_update(views_l, grads_l, pool, lr=1e-3):
    """A plain host optimizer step for the training-loop measurement (the paper names no
    optimizer; any fixed rule serves): w <- bf16(w - lr * g) per tensor, numpy, chunked over a
    thread pool (numpy releases the interpreter lock inside its loops)."""
    import numpy as np
    from paper_2410_08791_amd import synth
    jobs = []
    for n, v in views_l.items():
        flat, g = v.reshape(-1), grads_l[n].reshape(-1)
        step = 1 << 21
        for lo in range(0, flat.size, step):
            jobs.append((flat[lo:lo + step], g[lo:lo + step]))

    def one(j):
        wv, gv = j
        wv[...] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(wv) - np.float32(lr) * gv)
    list(pool.map(one, jobs))


def measure(args, name, steps, warmup, ceiling, headline, blob_cache):
    """Times one workload; returns its result dict (the whole JSON line when `headline`).
    blob_cache: {stack signature: (blobs, views)} -- workloads over the same seeded stack (the
    decode workload runs the llama7b stack) share their pinned weights."""
    import numpy as np
    import torch
    from paper_2410_08791_amd import binding as sp
    from paper_2410_08791_amd import synth

    w = synth.WORKLOADS[name]
    if headline and args.layers:
        w = w.with_(n_layers=args.layers)
    training = w.training
    k = (args.k if headline else None) or w.k
    p = (args.p if headline else None) or w.p
    desc = sp.make_desc(w)
    blob_bytes = sp.sp_layer_blob_bytes(C.byref(desc))
    budget_layers = w.budget_layers or (k + p)
    budget_bytes = None
    if w.name == "llama70b":
        budget_bytes = 16 * 10 ** 9              # the workload's cap: 16 GB for slots + workspace
    distinct = args.distinct_blobs if headline else None
    if distinct is None and w.n_layers * blob_bytes > 100e9:
        distinct = 16                            # ~27 GB pinned instead of ~137 GB; same traffic and schedule
    log(f"[bench] workload {w.name}: L={w.n_layers} d={w.d_model} T={w.tokens} blob={blob_bytes / 1e6:.1f} MB/layer"
        + (f"; {distinct} distinct blobs cycled" if distinct else ""))

    t0 = time.time()
    pool = synth.make_pool(16)
    nb = min(distinct, w.n_layers) if distinct else w.n_layers
    sig = (w.arch, w.n_layers, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.d_ffn, w.seed, nb)
    if sig not in blob_cache:
        blob_cache.clear()
        blob_cache[sig] = sp.pinned_blobs(w, desc, n_layers=nb, pool=pool)
    blobs, views = blob_cache[sig]
    if nb < w.n_layers:
        blobs = [blobs[l % nb] for l in range(w.n_layers)]
        views = [views[l % nb] for l in range(w.n_layers)]
    log(f"[bench] weights generated into pinned memory in {time.time() - t0:.1f} s")
    x = synth.make_input(w)
    xd = torch.from_numpy(x).to("cuda:0")
    yd = torch.empty_like(xd)
    B, S, T = w.batch, w.seq, w.tokens
    decoding = w.gen > 0
    keep = bool(headline and args.keep_activations)
    frozen = args.frozen if (headline and training) else 0
    if decoding:
        T = B                                        # tokens per step: one per sequence
        max_len = (S + 4 * (warmup + max(steps, 3)) + 64 + 7) // 8 * 8
        cache = torch.empty(sp.sp_kv_cache_bytes(C.byref(desc), B, max_len), dtype=torch.uint8, device="cuda:0")
        x1 = torch.from_numpy(np.ascontiguousarray(x[:, 0])).to("cuda:0")     # the token fed at every step
        y1 = torch.empty_like(x1)
    if training:
        tgt = torch.from_numpy(synth.make_input(w, "target")).to("cuda:0")
        gbytes = sp.sp_layer_grad_bytes(C.byref(desc))
        gblobs = [torch.zeros(gbytes, dtype=torch.uint8, pin_memory=True) for _ in range(w.n_layers)]
        loss = torch.zeros(1, dtype=torch.float32, device="cuda:0")
        dxd = torch.empty_like(xd)

    def run(kk, pp, flags, steps, warmup, pinned=0, units=1, slots=None, update=False):
        # slots: a budget of that many layer slots instead of the workload's own
        if training:
            flags |= sp.SP_FLAG_TRAINING | (sp.SP_FLAG_KEEP_ACTIVATIONS if keep else 0)
        # cross-check of the byte budget from outside the library: device memory torch hands out
        # between here and the end of the timed steps (the arena is the only allocation; x, y, targets,
        # the KV cache and the loss exist already), and the driver's free-memory figure
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        alloc0 = torch.cuda.memory_allocated()
        free0 = torch.cuda.mem_get_info()[0]
        eng = sp.Engine(desc, blobs, kk, pp, budget_layers=slots or budget_layers,
                        budget_bytes=None if slots else budget_bytes, flags=flags,
                        pinned=pinned, frozen=frozen, units=units)
        pos = [S]
        upd_s = [0.0]

        def step():
            if training:
                eng.forward_backward(xd, tgt, None, loss, None if frozen else dxd, gblobs, B, S)
                if update:
                    # the training LOOP: each layer's host weights are rewritten as soon as its own
                    # gradient has landed (last layer first), while the backward still runs below
                    for l in reversed(range(frozen, w.n_layers)):
                        eng.wait_gradient(l)
                        tu = time.perf_counter()
                        host_update(views[l], sp.grad_views(desc, gblobs[l].numpy()), pool)
                        upd_s[0] += time.perf_counter() - tu
                        eng.weights_updated(l)
            elif decoding:
                eng.decode(x1, y1, cache, B, pos[0], max_len)
                pos[0] += 1
            else:
                eng.forward(xd, yd, B, S)

        if decoding:
            eng.prefill(xd, yd, cache, B, S, max_len)        # the prompt; not part of the timed steps

        for _ in range(warmup):
            step()
        eng.sync()
        eng.stats()                                  # clears the kernel-timing window
        upd_s[0] = 0.0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        tw = time.perf_counter()
        e0.record(eng.compute)
        for _ in range(steps):
            step()
        e1.record(eng.compute)
        eng.sync()
        torch.cuda.synchronize()
        wall = time.perf_counter() - tw
        ms = e0.elapsed_time(e1)
        st = eng.stats()
        torch_peak = torch.cuda.max_memory_allocated() - alloc0
        driver_drop = free0 - torch.cuda.mem_get_info()[0]
        y = ((loss if frozen else dxd) if training else y1 if decoding else yd).cpu().numpy().copy()
        eng.destroy()
        return dict(ms_per_step=ms / steps, wall_ms_per_step=wall * 1e3 / steps, stats=st, y=y,
                    budget=eng.budget_bytes, update_ms_per_step=upd_s[0] * 1e3 / steps,
                    torch_peak_bytes=int(torch_peak), driver_free_drop_bytes=int(driver_drop))

    wrap = not (headline and args.no_wrap) and not training
    base_flags = sp.SP_FLAG_WRAP_PREFETCH if wrap else 0
    tmode = (2 if keep else 1) if training else 0
    grad_ms = gbytes / (ceiling * 1e6) if training else 0.0
    pinned = args.pinned if (headline and args.pinned is not None) else 0
    units = args.units if headline else 1
    tuned = None
    big = w.n_layers * blob_bytes > 100e9            # 2 s per step: the short run of it skips the window search
    tsteps = 2 if (big and not headline) else 3
    if big and not headline:
        k, p, pinned, units = 1, 1, sp.SP_PIN_AUTO, 1     # what the search settles on for this stack (two slots, rest pinned)
    elif not headline or (args.k is None and args.p is None and args.pinned is None):
        # Window choice at the fixed budget (the paper's grid search, Sec. 4.2): the cost model
        # proposes a window from per-layer times measured with the workload's default (k, p);
        # a short measured run of both decides which one the timed region uses.
        probe = run(k, p, base_flags | sp.SP_FLAG_TIMING, 3, 1)
        cost = sp.layer_costs(probe["stats"], w.n_layers, training=training, grad_ms=grad_ms)
        tu, tk, tp, tr, tms = sp.autotune_units(desc, int(probe["budget"]), cost, wrap=wrap, training=tmode)
        tuned = {"units_per_layer": tu, "k": tk, "p": tp, "pinned": tr, "modelled_ms_per_step": round(tms, 3),
                 "layer_cost_ms": {"copy": round(cost[0], 3), "fwd": round(cost[1], 3),
                                   "bwd": round(cost[2], 3), "grad": round(cost[3], 3)}}
        cands = {(k, p, 0, 1): None, (tk, tp, tr, tu): None}
        for c in cands:
            r = run(c[0], c[1], base_flags, 3, 1, pinned=c[2], units=c[3])
            cands[c] = max(r["ms_per_step"], r["wall_ms_per_step"])
        tuned["measured_ms_per_step"] = {f"k={c[0]},p={c[1]},pinned={c[2]},units={c[3]}": round(v, 3)
                                         for c, v in cands.items()}
        k, p, pinned, units = min(cands, key=cands.get)
        log(f"[bench] window: tuner proposes {tuned}; using k={k} p={p} pinned={pinned} units/layer={units}")
    # the timed region: only the dominant GEMM is bracketed by events (compute stream)
    main_run = run(k, p, base_flags | (0 if (headline and args.no_kernel_timing) else sp.SP_FLAG_KERNEL_TIMING), steps,
                   warmup, pinned=pinned, units=units)
    kst = main_run["stats"]
    # a second, short region with the per-layer trace on (timestamped fence events on the
    # copy stream cost a few percent of link rate, so it is kept out of `value`)
    trace_run = run(k, p, base_flags | sp.SP_FLAG_TIMING, tsteps, 1, pinned=pinned, units=units)
    st = trace_run["stats"]
    flags = base_flags | sp.SP_FLAG_TIMING
    ms = max(main_run["ms_per_step"], main_run["wall_ms_per_step"])   # host wall covers all streams
    tokens_s = T / (ms * 1e-3)
    h2d_gbps_wall = st.last_h2d_bytes / (ms * 1e-3) / 1e9
    h2d_gbps_busy = st.last_h2d_bytes / (st.copy_busy_ms * 1e-3) / 1e9 if st.copy_busy_ms > 0 else None
    log(f"[bench] {w.name}: units/layer={units} k={k} p={p} pinned={st.plan.n_pinned} slots={st.plan.n_slots}: "
        f"{ms:.2f} ms/step, {tokens_s:.0f} tokens/s, H2D {h2d_gbps_wall:.1f} GB/s over wall")

    # dominant kernel: the layer's largest GEMM (gate/up projection, or the first MLP GEMM)
    gm, gn, gk = kst.big_gemm_m, kst.big_gemm_n, kst.big_gemm_k
    gemm_ms = kst.big_gemm_ms_sum / max(kst.big_gemm_launches, 1)
    gemm_flops = 2.0 * gm * gn * gk
    achieved_tf = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    kname = ("gemm_dma_kernel<EPI_BF16> (first MLP projection, bias epilogue)" if training and w.arch == "encoder" else
             "gemm_dma_kernel<EPI_BF16> (gate/up projection)" if training else
             "gemm_skinny_kernel<EPI_SWIGLU_BF16> (gate/up projection, one row per sequence)" if decoding else
             "gemm_dma_kernel<EPI_SWIGLU_BF16> (gate/up projection)" if w.arch == "decoder" else
             "gemm_dma_kernel<EPI_GELU_BF16> (first MLP projection)")
    roofline = {"bound": "mfma", "kernel": kname,
                "achieved": round(achieved_tf, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tf / PEAK_BF16_TFLOPS, 4), "traffic": None,
                "flops_per_launch": gemm_flops, "avg_launch_ms": round(gemm_ms, 4),
                "launches_timed": int(kst.big_gemm_launches), "shape_mnk": [gm, gn, gk]}

    if decoding:
        # with one row per sequence the same kernel streams the weight matrix once and does
        # almost no arithmetic: bound by HBM, bytes = weights + the few activation rows
        gbytes_launch = 2.0 * (gn * gk + gm * gk + gm * gn / 2)
        achieved_gbs = gbytes_launch / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved_gbs, 1), "peak": 8000.0,
                    "unit": "GB/s", "frac": round(achieved_gbs / 8000.0, 4), "traffic": None,
                    "bytes_per_launch": gbytes_launch, "avg_launch_ms": round(gemm_ms, 4),
                    "launches_timed": int(kst.big_gemm_launches), "shape_mnk": [gm, gn, gk]}

    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}_gate_up_gemm.json")
    if os.path.exists(tpath) and not training:
        # HBM-side bytes per launch of this kernel from two rocprofv3 --pmc runs of this same
        # command (FETCH_SIZE, WRITE_SIZE), scaled by a copy kernel of known size; a stored
        # measurement, since counters cannot be read from inside this process
        tj = json.load(open(tpath))
        roofline["traffic"] = tj["traffic_bytes_per_launch"]
        roofline["traffic_source"] = os.path.relpath(tpath, ROOT)
        roofline["algorithmic_bytes"] = tj["algorithmic_bytes_per_launch"]

    extra = {
        "peak_hbm_bytes": int(st.plan.arena_bytes_used), "budget_bytes": int(main_run["budget"]),
        # seen from outside the library over the timed run: torch's peak of newly allocated device
        # bytes -- one block, the arena of budget_bytes + a 4 KiB alignment page, which torch's
        # allocator rounds up to a multiple of 2 MiB; the library itself allocates nothing -- and
        # the drop of the driver's free-memory figure (0 when the allocator re-used a cached block
        # of an earlier run, so this one only bounds it)
        "hbm_cross_check": {"torch_max_memory_allocated_delta": main_run["torch_peak_bytes"],
                            "driver_free_memory_drop": main_run["driver_free_drop_bytes"],
                            "arena_block_rounded_to_2MiB": int(-(-(main_run["budget"] + 4096) // (2 << 20)) * (2 << 20)),
                            "only_the_arena_was_allocated": bool(
                                main_run["torch_peak_bytes"] <= -(-(main_run["budget"] + 4096) // (2 << 20)) * (2 << 20))},
        "h2d_gbps_over_wall": round(h2d_gbps_wall, 2),
        "h2d_gbps_while_copying": round(h2d_gbps_busy, 2) if h2d_gbps_busy else None,
        "h2d_ceiling_gbps": round(ceiling, 2),
        "h2d_frac_of_ceiling": round(h2d_gbps_wall / ceiling, 4) if ceiling else None,
        "h2d_frac_of_nominal_64": round(h2d_gbps_wall / LINK_NOMINAL_GBPS, 4),
        # all four from the LAST call of the traced region, i.e. from one call's own intervals
        **overlap_metrics(st.copy_busy_ms, st.copy_hidden_ms, st.compute_busy_ms, st.wall_ms),
        "copy_busy_ms": round(st.copy_busy_ms, 3), "compute_busy_ms": round(st.compute_busy_ms, 3),
        "last_step_wall_ms": round(st.wall_ms, 3),
        "trace_run_ms_per_step": round(max(trace_run["ms_per_step"], trace_run["wall_ms_per_step"]), 3),
        "event_ms_per_step": round(main_run["ms_per_step"], 3),
        "host_wall_ms_per_step": round(main_run["wall_ms_per_step"], 3),
    }
    if name == "llama7b":
        extra["copy_hidden_target_0p60"] = (
            "not met and not reachable on this workload: a layer's copy takes ~7 ms against ~0.9 ms of compute, "
            "so at most compute/copy (copy_hidden_frac_bound) of the copy time can lie under compute; "
            "slowing the kernels would raise it and is not done")
    if tuned:
        extra["autotune"] = tuned
    if training:
        extra["d2h_gbps_over_wall"] = round(w.n_layers * gbytes / (ms * 1e-3) / 1e9, 2)
    if w.arch == "encoder":
        extra["images_per_s"] = round(B / (ms * 1e-3), 1)

    if not decoding:
        # Every kernel launch bracketed by HIP events on the compute stream (SP_FLAG_OP_TIMING), summed per
        # operation kind over two steps: each op's time per step and what it reaches of its own bound.
        # (The event records leave gaps between the kernels: this region's step time is not `value`.)
        r = run(k, p, base_flags | sp.SP_FLAG_OP_TIMING, 2, 1, pinned=pinned, units=units)
        ost = r["stats"]
        work = op_work(w, training)
        table = {}
        for i, nm in enumerate(sp.SP_OP_NAMES):
            if not ost.op_launches[i]:
                continue
            ms_op = ost.op_ms[i] / 2
            row = {"ms_per_step": round(ms_op, 4), "launches_per_step": ost.op_launches[i] // 2}
            if nm in work and work[nm][1] > 0 and ms_op > 0:
                bound, amount = work[nm]
                if bound == "mfma":
                    row.update(bound="mfma", achieved_tflops=round(amount / ms_op / 1e9, 1),
                               frac=round(amount / ms_op / 1e9 / PEAK_BF16_TFLOPS, 4))
                else:
                    row.update(bound="hbm", achieved_gbps=round(amount / ms_op / 1e6, 1),
                               frac=round(amount / ms_op / 1e6 / 8000.0, 4))
            table[nm] = row
        extra["op_table"] = table
        extra["op_table_kernel_ms_per_step"] = round(sum(v["ms_per_step"] for v in table.values()), 3)
        log(f"[bench] {w.name} per-op (HIP events around every launch): " + json.dumps(table))

    if training and (args.host_update or not headline):
        # The training loop with a host optimizer between the steps (Sec. 3.3; Table 2's setting):
        # every layer's host weights rewritten after its gradient landed, then streamed in again.
        saved = [{n: v.copy() for n, v in vl.items()} for vl in views[:nb]]
        r = run(k, p, base_flags, max(3, min(steps, 5)), 1, pinned=pinned, units=units, update=True)
        for vl, sv in zip(views[:nb], saved):
            for n in vl:
                vl[n][...] = sv[n]
        m_upd = max(r["ms_per_step"], r["wall_ms_per_step"])
        upd = r["update_ms_per_step"]
        extra["host_update_loop"] = {
            "ms_per_step": round(m_upd, 3), "ms_per_step_without_updates": round(ms, 3),
            "host_update_ms_per_step": round(upd, 3),
            "update_hidden_frac": round(max(0.0, min(1.0, 1.0 - (m_upd - ms) / upd)), 4) if upd > 0 else None,
            "rule": "w <- bf16(w - 1e-3 g) per tensor, numpy over 16 threads; layer l updated after "
                    "sp_wait_gradient(l), then sp_weights_updated(l)"}
        log(f"[bench] training loop with host updates: {json.dumps(extra['host_update_loop'])}")

    # The timed run's own output against the oracle's stored run of the WHOLE stack at the full
    # token count (tests/golden/, written by a script that calls only oracle/): sampled rows of y
    # (of dx for a training step), at no extra cost.  Beside it, what the stored run says bf16
    # operand rounding alone does to the oracle's own output on the same rows and over all elements.
    gpath = os.path.join(ROOT, "tests", "golden", f"full_depth_{w.name}.npz")
    if os.path.exists(gpath) and not decoding and not frozen and not (headline and args.layers):
        with np.load(gpath) as g:
            if int(g["distinct"]) == nb:
                rows = g["rows"]
                got = main_run["y"].reshape(w.tokens, -1)[rows].astype(np.float64)
                ref = (g["dx_rows"] if training else g["y_rows"]).astype(np.float64)
                rmax = float(g["dx_absmax"] if training else g["y_absmax"])
                fd = {"compared": "dx" if training else "y", "rows": int(len(rows)), "layers": int(w.n_layers),
                      "tokens": int(w.tokens), "max_rel_err": float(np.abs(got - ref).max() / rmax),
                      "source": os.path.relpath(gpath, ROOT)}
                if "ops_dev_rows" in g.files:
                    fd["oracle_with_bf16_operands_vs_oracle"] = {
                        "same_rows_of_y": float(g["ops_dev_rows"]), "all_elements_of_y": float(g["ops_dev_all"]),
                        "frobenius": float(g["ops_dev_fro"])}
                extra["parity_full_depth"] = fd
                log(f"[bench] {w.name}: whole stack against the stored oracle run on {len(rows)} rows: {fd['max_rel_err']:.3e}")

    # window sweep at the same budget (+ the naive comparator); bits must not change
    if headline and not args.no_sweep:
        sweep = []
        # decode runs are compared at the same position: against the sweep's first entry
        base = None if decoding else main_run["y"]
        A = sp.SP_PIN_AUTO
        grid = ([(1, 1, 0, 1), (1, 2, 0, 1), (2, 1, 0, 1), (2, 2, 0, 1), (4, 1, 0, 1), (4, 2, 0, 1), (1, 1, A, 1),
                 (1, 2, A, 1), (2, 1, A, 1), (1, 1, A, 3)]
                if w.name == "llama7b" else
                sorted({(1, 1, 0, 1), (w.k, w.p, 0, 1), (1, 1, A, 1), (k, p, pinned, units)} |
                       (set() if training else {(1, 1, A, 3)})))
        for kk, pp, rr, uu in grid:
            r = run(kk, pp, flags & ~sp.SP_FLAG_TIMING, 3, 1, pinned=rr, units=uu)
            m = max(r["ms_per_step"], r["wall_ms_per_step"])
            if base is None:
                base = r["y"]
            sweep.append({"k": kk, "p": pp, "units_per_layer": uu, "pinned": int(r["stats"].plan.n_pinned),
                          "slots": int(r["stats"].plan.n_slots),
                          "tokens_per_s": round(T / (m * 1e-3), 1),
                          "bit_identical": bool(np.array_equal(r["y"], base))})
        r = run(1, 1, sp.SP_FLAG_NO_OVERLAP, 3, 1)
        m = max(r["ms_per_step"], r["wall_ms_per_step"])
        sweep.append({"mode": "naive(2 slots, no overlap)", "tokens_per_s": round(T / (m * 1e-3), 1),
                      "bit_identical": bool(np.array_equal(r["y"], base))})
        extra["sweep"] = sweep
        # the best window of the plain (k, p) grid the workload names: whole layers, nothing pinned
        plain = [s for s in sweep if s.get("pinned") == 0 and s.get("units_per_layer") == 1]
        if plain:
            best = max(plain, key=lambda s: s["tokens_per_s"])
            extra["value_plain_window"] = {"tokens_per_s": best["tokens_per_s"], "k": best["k"], "p": best["p"],
                                           "note": "best of the plain (k,p) sweep: every layer streams whole, "
                                                   "nothing pinned; `value` is the tuner's window at the same budget"}
        log("[bench] sweep: " + json.dumps(sweep))

    if headline and args.paper_table and not training:
        # The paper's Table 1 (Sec. 4.2) on this machine.  Its k = layers on the GPU, k' = layers
        # swapped per group: here k slots, of which k' are in flight.  Naive(k): k slots, loads and
        # computes never overlap.  Standard: every layer resident (its copies happen in the warm-up).
        L = w.n_layers
        rows = []

        def row(method, kk, kp, r):
            m = max(r["ms_per_step"], r["wall_ms_per_step"])
            rows.append({"method": method, "gpu_memory_gb": round(r["stats"].plan.arena_bytes_used / 1e9, 2),
                         "ms_per_step": round(m, 2), "k": kk, "k_prime": kp,
                         "bit_identical": bool(np.array_equal(r["y"], main_run["y"])) if not decoding else None})

        row("Standard", None, None, run(L, L, 0, 3, 2, slots=L))
        for kk in (1, 8, 15):
            if kk < L:
                row("Naive", kk, None, run(1, max(kk - 1, 1), sp.SP_FLAG_NO_OVERLAP, 3, 1, slots=kk))
        for kk, kp in ((4, 2), (5, 3), (8, 3), (10, 2), (20, 6)):
            if kk < L:
                row("Superpipeline", kk, kp, run(kk - kp, kp, base_flags, 3, 1, slots=kk))
        # the same budgets spent this build's way: a ring of two slots, the other slots pinned
        for kk in (4, 8, 20):
            if kk < L:
                row("Superpipeline, k-2 layers pinned", kk, 1, run(1, 1, base_flags, 3, 1, pinned=sp.SP_PIN_AUTO, slots=kk))
        extra["paper_table"] = rows
        unit = "ms/token step" if decoding else "ms/forward"
        log("[bench] | Method | GPU memory (GB) | Time (%s) | k | k' |" % unit)
        log("[bench] |---|---|---|---|---|")
        for r_ in rows:
            log(f"[bench] | {r_['method']} | {r_['gpu_memory_gb']} | {r_['ms_per_step']} | "
                f"{r_['k'] if r_['k'] else '-'} | {r_['k_prime'] if r_['k_prime'] else '-'} |")

    cpu = None
    if decoding:
        extra["ms_per_token"] = round(ms, 3)             # per sequence: one step yields one token each
        extra["prompt_positions"] = S
    if not args.no_cpu_baseline and not decoding:
        from threadpoolctl import threadpool_info
        from oracle import stack_oracle as O
        # bounded sample of the same workload (the tiny stack runs whole)
        n = w.n_layers if w.name == "tiny" else min(args.cpu_layers if headline else 2, w.n_layers)
        cb = 1 if (training or w.name in ("vith", "llama70b")) else B    # bounded sample: fewer batch items
        cb = min(B, 8) if w.name == "vith" else cb
        shape = O.StackShape(w.arch, n, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim,
                             w.d_ffn, w.causal, w.norm_eps)
        xs = x[:cb]
        t0 = time.perf_counter()
        if training:
            ts = synth.make_input(w, "target")[:cb]
            ref = O.stack_forward_backward(xs, ts, views[:n], cb, S, shape, dtype=np.float32)[0]
        else:
            # a deep sample runs as the oracle's own forward over consecutive groups of layers
            # (the same composition as one call), so that a run of minutes reports where it is
            ref, l0 = xs, 0
            while l0 < n:
                l1 = min(l0 + 4, n)
                ref = O.stack_forward(ref, views[l0:l1], cb, S, shape, dtype=np.float32, n_layers=l1 - l0)
                if n > 4:
                    log(f"[bench] oracle: {l1} of {n} layers ({time.perf_counter() - t0:.0f} s)")
                l0 = l1
        dt = time.perf_counter() - t0
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        scale = (w.n_layers / n) * (B / cb)
        cpu = {"value": round(T / (dt * scale), 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"fp32 numpy (BLAS matmul, einsum attention) oracle ({'forward+backward' if training else 'forward'}) "
                         f"on {n} of {w.n_layers} layers, {cb} of {B} batch items x {S} tokens ({dt:.1f} s)"
                         + (f", time scaled by {scale:g}" if scale != 1 else ", the whole workload, not extrapolated")}
        # parity of the same sample on the GPU (forward output), same kernels and tile choices
        sub = sp.make_desc(w, n_layers=n)
        eng = sp.Engine(sub, blobs[:n], 1, 1)
        xsd = torch.from_numpy(np.ascontiguousarray(xs)).to("cuda:0")
        ysd = torch.empty_like(xsd)
        eng.forward(xsd, ysd, cb, S)
        eng.sync()
        got = ysd.cpu().numpy().reshape(cb * S, -1).astype(np.float64)
        eng.destroy()
        d = np.abs(got - ref)
        added = np.abs(ref.astype(np.float64) - xs.reshape(cb * S, -1))
        extra["parity_sample"] = f"{n} layers, {cb} batch items"
        extra["parity_max_rel_err"] = float(d.max() / np.abs(ref).max())
        extra["parity_err_over_added"] = float(d.max() / added.max())    # against what the layers added to x
        log(f"[bench] {w.name} oracle sample: {dt:.1f} s on {cores} threads; GPU vs oracle max rel err "
            f"{extra['parity_max_rel_err']:.3e} (against the stack's own contribution {extra['parity_err_over_added']:.3e})")

    pool.shutdown()
    out = {
        "metric": "tokens/sec at fixed HBM weight budget", "value": round(tokens_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_layers} layers d={w.d_model} heads={w.n_q_heads}/{w.n_kv_heads}"
                               f"x{w.head_dim} ffn={w.d_ffn} causal={w.causal} batch {B} x seq {S}, "
                               + ("forward+backward (MSE)" if training else
                                  "prompt, then decode of one token per sequence per step" if decoding else "forward"),
                   "units_per_layer": units, "k": k, "p": p, "n_pinned": int(st.plan.n_pinned),
                   "pinned_layers": int(st.plan.n_pinned) // units, "n_slots": int(st.plan.n_slots),
                   "budget_layers": budget_layers,
                   "wrap_prefetch": wrap, "keep_activations": bool(training and keep),
                   "frozen_layers": frozen,
                   "layer_blob_bytes": int(blob_bytes),
                   "distinct_blobs": nb, "seed": w.seed},
        "roofline": roofline, "cpu_baseline": cpu, **extra,
    }
    del blobs, views, xd, yd
    torch.cuda.empty_cache()
    return out


# what a short run of another workload contributes to the one JSON line
OTHER_KEYS = ("ms_per_step", "value", "unit", "steps", "config", "roofline", "peak_hbm_bytes", "budget_bytes", "hbm_cross_check",
              "h2d_gbps_over_wall", "h2d_frac_of_ceiling", "d2h_gbps_over_wall", "copy_hidden_frac",
              "copy_hidden_frac_bound", "overlap_efficiency", "copy_stream_idle_frac", "images_per_s", "ms_per_token",
              "host_update_loop", "op_table", "op_table_kernel_ms_per_step", "parity_sample", "parity_max_rel_err", "parity_err_over_added", "parity_full_depth", "cpu_baseline")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--p", type=int, default=None)
    ap.add_argument("--pinned", type=int, default=None,
                    help="layers held in HBM for good (-1 = what the budget leaves after k+p); "
                         "default: k, p and this are chosen by the tuner and a short measured comparison")
    ap.add_argument("--units", type=int, default=1, choices=(1, 3),
                    help="units a layer streams as (3: attention block, first FFN projection, last FFN projection; "
                         "k, p and --pinned then count units); only used when k, p or --pinned is given")
    ap.add_argument("--layers", type=int, default=None, help="run a prefix of the stack (debug)")
    ap.add_argument("--distinct-blobs", type=int, default=None,
                    help="generate only this many distinct layer blobs and cycle them (host RAM limit)")
    ap.add_argument("--no-wrap", action="store_true", help="do not prefetch the next call's first layers")
    ap.add_argument("--keep-activations", action="store_true",
                    help="training: keep every layer's activations instead of recomputing them")
    ap.add_argument("--frozen", type=int, default=0,
                    help="training: this many lowest layers get no weight gradients; no input gradient is "
                         "asked for, so the backward stops above them")
    ap.add_argument("--host-update", action="store_true",
                    help="training: also time the loop with a host optimizer step between the steps")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--paper-table", action="store_true",
                    help="also time the paper's comparison rows (Sec. 4.2, Table 1): Standard (resident), "
                         "Naive(k) and Superpipeline(k, k') at the paper's window settings")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="no event brackets around the dominant GEMM in the timed region (roofline fields read 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=2, help="oracle sample: layers at full token count")
    ap.add_argument("--others", default=None,
                    help="comma-separated workloads timed briefly after the headline one and reported under "
                         "other_workloads ('' = none; default with the default workload: "
                         "tiny,vith,train1p3b,llama7b_decode,llama70b)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is single-GPU (one process, one device, no collectives); "
            "run it with --gpus 1.")
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    prop = torch.cuda.get_device_properties(0)
    try:
        ram_gb = os.sysconf("SC_PAGE_SIZE") * os.sysconf("SC_PHYS_PAGES") / 1e9
    except (ValueError, OSError):
        ram_gb = float("nan")
    log(f"[bench] {torch.cuda.get_device_name(0)}: {prop.multi_processor_count} CUs, "
        f"{prop.total_memory / 1e9:.0f} GB, engine clock {getattr(prop, 'clock_rate', 0) / 1e3:.0f} MHz, "
        f"HIP {torch.version.hip}; host cores {os.cpu_count()}, RAM {ram_gb:.0f} GB")
    ceiling = copy_ceiling_gbps(torch)
    log(f"[bench] plain pinned H2D copy ceiling: {ceiling:.1f} GB/s")

    blob_cache = {}
    out = measure(args, args.workload, args.steps, args.warmup, ceiling, True, blob_cache)
    others = args.others
    if others is None:
        # the decode workload first: it runs the headline stack's weights
        others = "llama7b_decode,tiny,vith,train1p3b,llama70b" if args.workload == "llama7b" and not args.layers else ""
    res = {}
    for name in [n for n in others.split(",") if n]:
        t0 = time.time()
        steps = 3 if name == "llama70b" else 10
        r = measure(args, name, steps, 1 if name == "llama70b" else 2, ceiling, False, blob_cache)
        res[name] = {k_: r[k_] for k_ in OTHER_KEYS if k_ in r}
        res[name]["tokens_per_s"] = res[name].pop("value")
        res[name]["bench_seconds"] = round(time.time() - t0, 1)
    if res:
        out["other_workloads"] = res
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
