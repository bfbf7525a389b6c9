#!/usr/bin/env python3
"""Benchmark of the braided F/B/W units of one TP shard on one MI355X.

A "step" is one braided execution block (paper Section 3, Fig. 3a): the four forward units
of microbatch 1 interleaved with the full backward (B and W units) of microbatch 0 of the
same layer, on three HIP streams.  One step therefore performs exactly the F + B + W work of
one layer-microbatch.  Headline workload: GPT-7B-style layer, TP=8 shard (hidden 4096, 4 of 32
heads x 128, FFN shard 2048), sequence 6144, microbatch 1, bf16 storage with fp32 accumulation.

The defaults time 200 steps after 20 warm-up steps: after an idle period the chip needs some tens of
milliseconds to reach its steady clocks (30 timed steps read 4 % slower than 200 or 1000, which agree), and a
training loop runs in the steady state.  The single-kernel legs repeat their launches as often for the same reason.

Prints one JSON line (see the repository's design notes for the field definitions).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak (256 CU x 4096 flop/clk x 2.4 GHz ~ 2.5e15)
# HBM-side bytes per launch of the dominant kernel on its four shapes, from the two rocprofv3 --pmc runs
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors calibrated on a 1 GiB copy) summarised in the file named below;
# counters cannot be read from inside this process, so this is a recorded figure, not one this run measured.
GEMM_FWD_TRAFFIC_BYTES = 177.9e6
GEMM_FWD_TRAFFIC_SOURCE = "profiles/gemm_bf16_fwd_layout_gpt7b_tp8.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --only-gemm`; a constant recorded from that profile, not measured by this run)"


def unit_flops(wl):
    """Algorithmic flops of the F, B and W units of one layer-microbatch: GEMMs as 2MNK; causal
    attention counts only the unmasked pairs s(s+1)/2; attention backward counts its four
    matmuls (no recomputation)."""
    T, h, a, f = wl.seq, wl.hidden, wl.attn_local, wl.ffn_local
    pairs = T * (T + 1) // 2 if wl.causal else T * T
    n_in = 2 if wl.act == "swiglu" else 1
    qkv, outp = 2 * T * h * wl.qkv_local, 2 * T * a * h      # QKV width: Q heads + 2 x key / value heads
    fc1, fc2 = n_in * 2 * T * h * f, 2 * T * f * h
    F = qkv + 4 * a * pairs + outp + fc1 + fc2
    B = fc2 + fc1 + outp + 8 * a * pairs + qkv
    W = fc2 + fc1 + outp + qkv
    return {"F": F, "B": B, "W": W, "gemm_fwd": [qkv, outp, fc1 // n_in, fc2]}


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_each(fn, reps, warmup, torch):
    """Mean time of `reps` runs of fn, each between two device synchronisations of its own (a whole sequence
    with its copies to and from the host, as one training iteration would run it)."""
    for _ in range(warmup):
        fn()
    total = 0.0
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
    return total * 1e3 / reps


def event_steps(ctx, stage, arr, streams, steps, torch):
    """Per-step makespans of `steps` braided steps from HIP events: after every step a timing stream waits for
    the step's end on all three streams and records an event; a step's time is the distance between two such
    events (the next step waits for the same three ends, so the steps do not overlap).  Returns the list in ms."""
    sF, sB, sW = streams
    sT = torch.cuda.Stream()
    marks = []

    def mark():
        for s in (sF, sB, sW):
            e = torch.cuda.Event()
            e.record(s)
            sT.wait_event(e)
        m = torch.cuda.Event(enable_timing=True)
        m.record(sT)
        marks.append(m)

    for _ in range(3):
        ctx.braid_step(stage, arr, sF, sB, sW)
    mark()
    for _ in range(steps):
        ctx.braid_step(stage, arr, sF, sB, sW)
        mark()
    torch.cuda.synchronize()
    return [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]


GEMM_SHAPE_OVERRIDE = None     # --gemm-shape M,N,K: one shape instead of the workload's four (with --only-gemm)


def gemm_shapes(wl):
    if GEMM_SHAPE_OVERRIDE:
        return [GEMM_SHAPE_OVERRIDE]
    return [(wl.seq, wl.qkv_local, wl.hidden), (wl.seq, wl.hidden, wl.attn_local),
            (wl.seq, wl.ffn_local, wl.hidden), (wl.seq, wl.hidden, wl.ffn_local)]


def gemm_operands(shape, td, operands, torch):
    """A [M, K] and B [K, N]: N(0,1) activations against N(0, 0.02) weights, or all zeros.  The MFMA rate this
    chip sustains depends on the operand bits (power management slows the shader clock when the multipliers toggle
    on every bit), so a figure must say which data it ran on: the zeros leg shows what the same instruction stream
    reaches when power does not limit it."""
    M, N, K = shape
    if operands == "zeros":
        return torch.zeros((M, K), device="cuda", dtype=td), torch.zeros((K, N), device="cuda", dtype=td)
    return torch.randn((M, K), device="cuda").to(td), (torch.randn((K, N), device="cuda") * 0.02).to(td)


def gemm_leg(ctx, wl, reps, torch, stp, operands="random", library=False, per_shape=False):
    """Dominant kernel: the bf16 MFMA GEMM in its forward layout (A row-major, B = W[in,out]).  Its four
    launches per step (QKV, out-proj, FC1, FC2 shapes of the workload) are replayed alone on the current
    stream between HIP events recorded on that same stream.  Returns (average ms per launch, average
    algorithmic flops per launch), or the per-shape times in ms with `per_shape`.  With `library` the same
    shapes and operands go through torch.matmul (the vendor GEMM library) instead: a point of comparison that is
    reported beside the kernel's figure, never part of the path."""
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    code = stp.BF16 if wl.dtype == "bf16" else stp.F32
    shapes = gemm_shapes(wl)
    runs = []
    for (M, N, K) in shapes:
        A, Bm = gemm_operands((M, N, K), td, operands, torch)
        Cm = torch.empty((M, N), device="cuda", dtype=td)
        if library:
            runs.append((lambda A=A, Bm=Bm, Cm=Cm: torch.matmul(A, Bm, out=Cm)))
        else:
            g = stp.GemmArgs(dtype=code, M=M, N=N, K=K, A=A.data_ptr(), lda=K, B=Bm.data_ptr(), ldb=N,
                             C=Cm.data_ptr(), ldc=N, bias_scale=1.0, resid_scale=1.0)
            runs.append((lambda g=g, keep=(A, Bm, Cm): ctx.gemm(g)))
    for _ in range(3 if library else 1):
        for run in runs:
            run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if per_shape:
        out = []
        for run in runs:
            e0.record()
            for _ in range(reps):
                run()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / reps)
        return out
    e0.record()
    for _ in range(reps):
        for run in runs:
            run()
    e1.record()
    torch.cuda.synchronize()
    avg_ms = e0.elapsed_time(e1) / (reps * len(runs))
    return avg_ms, sum(2 * M * N * K for (M, N, K) in shapes) / len(shapes)


def gemm_context(ctx, wl, reps, torch, stp):
    """What frames the dominant kernel's figure: the same four launches on all-zero operands, and the vendor
    library's GEMM on both kinds of operands."""
    out = {"operands_of_achieved": "A ~ N(0,1), B ~ N(0,0.02), bf16"}
    for operands in ("zeros", "random"):
        for library in (False, True):
            if operands == "random" and not library:
                continue
            ms, fl = gemm_leg(ctx, wl, reps, torch, stp, operands=operands, library=library)
            key = ("library_" if library else "this_kernel_") + operands
            out[key] = {"avg_launch_ms": ms, "achieved": fl / (ms * 1e-3) / 1e12,
                        "frac": fl / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
    out["library"] = "torch.matmul(out=) on the same shapes, bf16 (the vendor GEMM library; comparison only)"
    return out


HBM_PEAK_GBS = 8000.0
HOST_LINK_BPS = 50e9          # device <-> page-locked host memory, one direction, large copies (measured 54 - 55 GB/s)


def hbm_leg(ctx, wl, torch, stp, reps=200):
    """The HBM-bound kernels of the units at the workload's sizes, alone on the current stream: achieved
    GB/s = algorithmic bytes (each tensor read or written once) / HIP-event time.  At these sizes (25-200 MB)
    part of the traffic is served by the 256 MB last-level cache, so a figure can exceed what HBM alone gives."""
    T, h, f, a = wl.seq, wl.hidden, wl.ffn_local, wl.attn_local
    td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    es = 2 if wl.dtype == "bf16" else 4
    code = stp.BF16 if wl.dtype == "bf16" else stp.F32
    norm = stp.NORM_LN if wl.norm == "ln" else stp.NORM_RMS
    mk = lambda *shape: torch.randn(*shape, device="cuda").to(td)
    x, dy, dr, y = mk(T, h), mk(T, h), mk(T, h), torch.empty((T, h), device="cuda", dtype=td)
    g, b = torch.ones(h, device="cuda").to(td), torch.zeros(h, device="cuda").to(td)
    stats = torch.empty((T, 2), device="cuda")
    dg, db, outb = torch.zeros(h, device="cuda"), torch.zeros(h, device="cuda"), torch.zeros(h, device="cuda")
    rsum = torch.zeros(h, device="cuda")
    hh, hd, hy = mk(T, f), mk(T, f), torch.empty((T, f), device="cuda", dtype=td)
    legs = [
        ("norm_fwd", 2 * T * h * es, lambda: ctx.norm_forward(code, norm, T, h, wl.eps, x, g, b, y, stats)),
        ("norm_bwd_resid_dgamma", 4 * T * h * es,
         lambda: ctx.norm_backward(code, norm, T, h, x, g, stats, dy, dr, y, dg, db)),
        # as the Pre-* B units run it: the row-parallel bias gradient (column sum of the residual-path gradient) rides along
        ("norm_bwd_resid_dgamma_biasgrad", 4 * T * h * es,
         lambda: ctx.norm_backward(code, norm, T, h, x, g, stats, dy, dr, y, dg, db, d_resid_sum=rsum, d_resid_sum_scale=0.125)),
        ("gelu_fwd", 2 * T * f * es, lambda: ctx.gelu_forward(code, T * f, hh, hy)),
        ("gelu_bwd", 3 * T * f * es, lambda: ctx.gelu_backward(code, T * f, hh, hd, hy)),
        ("swiglu_fwd", 3 * T * f * es, lambda: ctx.swiglu_forward(code, T * f, hh, hd, hy)),
        ("softmax_fwd_T_h", 2 * T * h * es, lambda: ctx.softmax_forward(code, T, h, 0.125, False, x, y)),
        ("softmax_bwd_T_h", 3 * T * h * es, lambda: ctx.softmax_backward(code, T, h, 0.125, x, dy, y)),
        ("colsum_T_h", T * h * es, lambda: ctx.colsum(code, T, h, x, 1.0, outb)),
        ("colsum_T_f", T * f * es, lambda: ctx.colsum(code, T, f, hh, 1.0, outb[:f])),
        # the practical ceiling: plain device copies of the same sizes (tensors of 25-100 MB are partly served by
        # the 256 MB last-level cache) and of 1 GiB (HBM alone)
        ("device_copy_T_h", 2 * T * h * es, lambda: y.copy_(x)),
        ("device_copy_T_f", 2 * T * f * es, lambda: hy.copy_(hh)),
        ("device_copy_1GiB", 2 << 30, lambda: big_dst.copy_(big_src)),
    ]
    big_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    big_dst = torch.empty_like(big_src)
    out = {}
    for name, nbytes, fn in legs:
        for _ in range(20):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = nbytes / ms / 1e6
        out[name] = {"us": ms * 1e3, "GB/s": gbs, "frac_of_8TBs": gbs / HBM_PEAK_GBS, "bytes": nbytes}
    return out


def attention_leg(ctx, wl, torch, stp, reps=200):
    """The attention core alone at the workload's shape (Attention(.) of Eq. 1 and its backward pass): forward call
    (main kernel + combine) and backward call (row dot, dK/dV and dQ kernels, combines), HIP events on the launching
    stream.  Rates count the algorithmic products only: 2 per unmasked (query, key) pair and head dimension forwards
    (S and PV), 4 backwards (dV, dP, dQ, dK); the backward kernels execute 7 for those 4 plus the forward's S."""
    T, n, d = wl.seq * 1, wl.heads_local, wl.head_dim
    desc = stp.make_desc(wl)
    bf = torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(11)
    qkv = (torch.randn(T, wl.qkv_local, device="cuda", generator=g) * 0.5).to(bf)
    dout = torch.randn(T, n * d, device="cuda", generator=g).to(bf)
    out = torch.empty(T, n * d, device="cuda", dtype=bf)
    lse = torch.empty(n * T, device="cuda", dtype=torch.float32)
    delta = torch.empty(n * T, device="cuda", dtype=torch.float32)
    dqkv = torch.empty_like(qkv)
    nkv = getattr(wl, "kv_heads", 0) or n
    pairs = T * (T + 1) / 2 if desc.causal else float(T) * T
    fwd_flops = 4.0 * pairs * d * n

    def timed(fn):
        for _ in range(max(10, reps // 10)):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_f = timed(lambda: ctx.attention_forward(desc, qkv, out, lse))
    ms_b = timed(lambda: ctx.attention_backward(desc, qkv, out, lse, dout, delta, dqkv))
    return {"forward_ms": ms_f, "forward_tflops": fwd_flops / (ms_f * 1e-3) / 1e12,
            "backward_ms": ms_b, "backward_tflops_algorithmic": 2.0 * fwd_flops / (ms_b * 1e-3) / 1e12,
            "shape": f"{n} query heads x {d}, {nkv} key/value heads, seq {T}, causal {int(desc.causal)}, bf16",
            "how": f"each call alone on the GPU, {reps} in a row between HIP events, random operands"}


def cpu_baseline(wl, w_host, fl, synth, reps=1):
    """The fp64 oracle on the host cores: the F, B and W units of one layer-microbatch of `wl`, timed apart."""
    import numpy as np
    from oracle import stp_oracle as O
    cfg = O.LayerCfg(hidden=wl.hidden, heads_local=wl.heads_local, head_dim=wl.head_dim, ffn_local=wl.ffn_local, tp=wl.tp,
                     norm=wl.norm, act=wl.act, causal=wl.causal, rope=wl.rope, has_bias=wl.has_bias,
                     eps=wl.eps, rope_base=wl.rope_base, kv_heads_local=wl.kv_heads)
    W64 = {k: v.astype(np.float64) for k, v in w_host.items()}
    X = synth.make_activation(wl, 0, "x.mb0").astype(np.float64)
    dO = synth.make_activation(wl, 0, "dy.mb0").astype(np.float64)
    tF = tB = tW = 0.0
    for _ in range(reps):
        st, g = {}, {}
        t0 = time.perf_counter()
        O.forward_unit(cfg, O.PRE_ATTN, W64, st, x_in=X)
        xa = O.forward_unit(cfg, O.ATTN, W64, st, x_resid=X)
        O.forward_unit(cfg, O.PRE_MLP, W64, st, x_in=xa)
        O.forward_unit(cfg, O.MLP, W64, st, x_resid=xa)
        t1 = time.perf_counter()
        dz = O.backward_input_unit(cfg, O.MLP, W64, st, dO)
        dxa = O.backward_input_unit(cfg, O.PRE_MLP, W64, st, dz, d_resid=dO, grads=g)
        dxl = O.backward_input_unit(cfg, O.ATTN, W64, st, dxa)
        O.backward_input_unit(cfg, O.PRE_ATTN, W64, st, dxl, d_resid=dxa, grads=g)
        t2 = time.perf_counter()
        O.backward_weight_unit(cfg, O.MLP, st, dO, g)
        O.backward_weight_unit(cfg, O.ATTN, st, dxa, g)
        t3 = time.perf_counter()
        tF, tB, tW = tF + (t1 - t0) / reps, tB + (t2 - t1) / reps, tW + (t3 - t2) / reps
    total = fl["F"] + fl["B"] + fl["W"]
    return {"value": total / (tF + tB + tW) / 1e12, "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
            "kind": "oracle",
            "sample": f"one full layer-microbatch (F, B and W units, all of a step's work) of workload {wl.name} in numpy fp64"
                      + (f", mean of {reps} passes" if reps > 1 else ""),
            "seconds": tF + tB + tW,
            "units": {"F": {"seconds": tF, "tflops": fl["F"] / tF / 1e12}, "B": {"seconds": tB, "tflops": fl["B"] / tB / 1e12},
                      "W": {"seconds": tW, "tflops": fl["W"] / tW / 1e12}}}


def stage_bench(ctx, args, torch, stp, synth):
    """Makespan of one stage's braided unit sequence (warm-up F, F&B with W separated, F&W, steady F&BW,
    degraded BW / B, cool-down W) against the same sequence on one stream and the sum of isolated units."""
    from paper_2510_27257_amd.binding import OP_B
    from paper_2510_27257_amd.stage import StageOnDevice, backward_ops, forward_ops, stage_sequence, weight_ops
    lm = synth.WORKLOADS["gpt7b_tp8_s4096"]
    if args.stage == "pp4":
        layers, cb = [lm] * 4, None
    else:
        layers, cb = [synth.WORKLOADS["vit"]] * 2 + [lm] * 2, [0, 0, 1, 0, 0]
    n_mb = 8
    stg = StageOnDevice(ctx, layers, n_mb, seed=0, chain_break=cb, tuned_tiles=not args.no_tuned_tiles)
    stg.load_inputs()
    L = len(layers)
    sched = None
    if args.schedule:
        # one device's program of the p-device schedule (Section 4.2), the stage split into its two chunks
        from paper_2510_27257_amd import schedule as S
        p_, m_, d_ = (int(x) for x in args.schedule.split(","))
        fl0 = unit_flops(layers[0])
        tt = S.Times(TF=fl0["F"], TB=fl0["B"], TW=fl0["W"], TAR=0.0)      # relative block lengths: the flop counts
        progs = S.build(p_, m_, steady_w_tail=args.schedule_w_tail)
        S.simulate(p_, progs, tt)
        n_mb = m_
        first1 = cb.index(1) if cb and 1 in cb else L // 2
        if cb is None:
            cb = [0] * (L + 1)
            cb[first1] = 1
        stg = StageOnDevice(ctx, layers, n_mb, seed=0, chain_break=cb, tuned_tiles=not args.no_tuned_tiles)
        stg.load_inputs()
        step_lists = S.braid_steps(progs[d_], L, first1)
        seq_name = f"program of device {d_} of {p_} ({m_} microbatches) from the schedule generator"
        mt = S.metrics(p_, progs, tt)[d_]
        sched = {"p": p_, "m": m_, "device": d_, "blocks": len(progs[d_]), "steady_w_tail": args.schedule_w_tail,
                 "simulated_peak_with_w_stashes": mt["peak_with_w_stash"],
                 "simulated_peak_activations": mt["peak_activation"], "table1_peak_activations": 3 * p_,
                 "plain_forward_blocks": sum(1 for b in progs[d_] if b.f and not b.b and not b.w)}
    elif args.pattern:
        from paper_2510_27257_amd.stage import two_chunk_sequence
        first1 = cb.index(1) if cb and 1 in cb else L // 2          # chunk 1 starts at the chain break
        step_lists = two_chunk_sequence(L, first1, n_mb, args.pattern)
        seq_name = f"two chunks (layers 0-{first1 - 1} | {first1}-{L - 1}), pairing pattern {args.pattern}"
    else:
        step_lists = stage_sequence(L, n_mb, warmup=args.stage_warmup)
        seq_name = f"three-phase sequence, {args.stage_warmup} forward pass(es) before the first backward"
    from paper_2510_27257_amd.stage import peak_in_flight
    peak = peak_in_flight(step_lists, L)
    steps = [(stp.Op * len(st))(*st) for st in step_lists]
    sF, sB, sW = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    s0 = torch.cuda.current_stream()
    off = None
    if args.offload_alpha is not None:
        from paper_2510_27257_amd.stage import Offloader
        off = Offloader(stg)          # its copy streams are created next to the compute streams

    def run(streams):
        ctx.braid_reset()
        for arr in steps:
            ctx.braid_step(stg.stage, arr, *streams)

    reps = max(3, min(10, args.steps // 6))
    ms_braided = time_steps(lambda: run((sF, sB, sW)), reps, 1, torch)
    ms_serial = time_steps(lambda: run((s0, s0, s0)), reps, 1, torch)
    # isolated units, per layer kind: F, B, W of one layer-microbatch alone on one stream
    ctx.braid_reset()
    ctx.braid_step(stg.stage, (stp.Op * (4 * L))(*forward_ops(L, 0)), s0, s0, s0)
    ctx.braid_step(stg.stage, (stp.Op * (4 * L))(*backward_ops(L, 0, OP_B)), s0, s0, s0)
    torch.cuda.synchronize()
    sum_iso, flops = 0.0, 0
    for l in range(L):
        f_ops = (stp.Op * 4)(*[o for o in forward_ops(L, 0) if o.layer == l])
        b_ops = (stp.Op * 4)(*[o for o in backward_ops(L, 0, OP_B) if o.layer == l])
        w_ops = (stp.Op * 2)(*[o for o in weight_ops(L, 0) if o.layer == l])
        for ops in (f_ops, b_ops, w_ops):
            sum_iso += n_mb * time_steps(lambda: ctx.braid_step(stg.stage, ops, s0, s0, s0), 10, 2, torch)
        fl = unit_flops(layers[l])
        flops += n_mb * (fl["F"] + fl["B"] + fl["W"])
    offload = None
    if args.offload_alpha is not None:
        # Section 4.2 / 4.3: a share alpha of the long-lived stashes goes to page-locked host memory on a copy
        # stream and comes back before its consumer; the paper's condition is T_o < T_F per model chunk
        from paper_2510_27257_amd.binding import OFFLOAD_FWD, OFFLOAD_W_ATTN as B_W_ATTN, OFFLOAD_W_MLP as B_W_MLP
        from paper_2510_27257_amd.stage import run_sequence_with_offload
        alpha = args.offload_alpha
        moved = [0]
        # a reload has to be under way for as long as its copy takes: per microbatch the stashes of all layers,
        # at the link's rate, in steps of the sequence's average length
        if args.offload_lead > 0:
            lead = args.offload_lead
        else:
            per_mb = 0
            if args.offload_sets in ("fwd", "both"):
                per_mb = max(per_mb, sum(off.bytes(l, OFFLOAD_FWD, alpha) for l in range(L)))
            if args.offload_sets in ("w", "both"):
                per_mb = max(per_mb, sum(off.bytes(l, B_W_MLP, alpha) + off.bytes(l, B_W_ATTN, alpha) for l in range(L)))
            lead = max(1, math.ceil(per_mb / HOST_LINK_BPS / (ms_braided * 1e-3 / len(steps))))

        def run_off():
            ctx.braid_reset()
            moved[0] = run_sequence_with_offload(ctx, stg, steps, (sF, sB, sW), off, alpha,
                                                 forward_stash=args.offload_sets in ("fwd", "both"),
                                                 w_stash=args.offload_sets in ("w", "both"),
                                                 min_gap=args.offload_min_gap, lead=lead)

        # every sequence between synchronisations of its own: issued back to back, the host blocks inside the
        # asynchronous copy calls of the next sequence while the previous one's copies are in flight (measured:
        # 35 ms per sequence against 29.7 ms for one alone), which is the runtime's doing and no part of a
        # training iteration, which ends in a synchronisation anyway
        ms_off = time_each(run_off, reps, 1, torch)
        ms_plain_each = time_each(lambda: run((sF, sB, sW)), reps, 1, torch)
        # T_o: the forward stash of the whole chunk (all layers, one microbatch), copied alone
        def copy_alone():
            for l in range(L):
                off.offload(l, 0, OFFLOAD_FWD, alpha, off.copy_stream)
        ms_to = time_steps(copy_alone, 5, 1, torch)
        f_all = (stp.Op * (4 * L))(*forward_ops(L, 0))
        ms_tf = time_steps(lambda: ctx.braid_step(stg.stage, f_all, s0, s0, s0), 5, 1, torch)
        chunk_bytes = sum(off.bytes(l, OFFLOAD_FWD, alpha) for l in range(L))
        offload = {"alpha": alpha, "sets": args.offload_sets, "min_gap_steps": args.offload_min_gap, "reload_lead_steps": lead,
                   "makespan_ms": ms_off, "makespan_without_ms": ms_plain_each,
                   "timing": "each sequence between device synchronisations of its own",
                   "bytes_to_host_per_sequence": moved[0], "bytes_back_per_sequence": moved[0],
                   "T_o_ms_forward_stash_of_chunk": ms_to, "T_F_ms_chunk": ms_tf,
                   "d2h_GBps": chunk_bytes / ms_to / 1e6 if ms_to > 0 else None,
                   "T_o_below_T_F": ms_to < ms_tf}
    print(json.dumps({
        "metric": "braided stage sequence TFLOP/s", "value": flops / (ms_braided * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": ms_braided, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"stage {args.stage}: {L} layers x {n_mb} microbatches, sequence of {len(steps)} braided blocks",
                   "sequence": seq_name, "peak_layer_stashes_in_flight": peak, "flops_per_step": flops,
                   "gemm_tile_hints": ((f"{stg.n_tile_hints} measured tile preferences of paper_2510_27257_amd/tuned_tiles.json, "
                                        f"objective '{stg.tuned_objective}' (a stage's sequence of steps)") if stg.n_tile_hints
                                       else ("none: on a stage's sequence of steps the library's own tile choice measured best for these layers "
                                             "(paper_2510_27257_amd/tuned_tiles.json)") if stg.tuned
                                       else "none (the library's own tile choice)")},
        "braid": {"makespan_ms": ms_braided, "serialized_ms": ms_serial, "sum_isolated_ms": sum_iso,
                  "makespan_over_sum_isolated": ms_braided / sum_iso},
        "offload": offload, "schedule": sched}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt7b_tp8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tuned-tiles", action="store_true",
                    help="leave the measured GEMM tile preferences of the package's tuned_tiles.json aside")
    ap.add_argument("--stage", choices=["pp4", "mllm"], default=None,
                    help="time one pipeline stage's whole braided sequence instead of the single block: "
                         "pp4 = 4 GPT-7B TP=8 layers at seq 4096, 8 microbatches; mllm = 2 ViT layers + 2 such "
                         "LM layers, 8 microbatches")
    ap.add_argument("--stage-warmup", type=int, default=1,
                    help="with --stage: forward passes in flight before the first backward pass (1 = memory-efficient "
                         "warm-up, more = throughput-efficient warm-up)")
    ap.add_argument("--schedule-w-tail", type=int, default=0,
                    help="with --schedule: the last N braids of the steady phase store their W (Section 4.2)")
    ap.add_argument("--schedule", default=None, metavar="P,M,D",
                    help="with --stage: replay the program of device D of the P-device, M-microbatch schedule "
                         "(the stage is split into two model chunks)")
    ap.add_argument("--pattern", type=int, choices=[1, 2], default=None,
                    help="with --stage: treat the stage as two model chunks and pair forward and backward units of "
                         "the same chunk (2) or of different chunks (1)")
    ap.add_argument("--offload-alpha", type=float, default=None,
                    help="with --stage: also time the sequence with a share alpha of the long-lived stashes "
                         "offloaded to page-locked host memory and reloaded (reported under \"offload\")")
    ap.add_argument("--offload-min-gap", type=int, default=1,
                    help="move only stashes whose consumer is at least this many braid steps after their producer")
    ap.add_argument("--offload-lead", type=int, default=0,
                    help="with --offload-alpha: steps a reload is enqueued ahead of its consumer (0 = as many as the copy "
                         "takes at 50 GB/s)")
    ap.add_argument("--offload-sets", choices=["w", "fwd", "both"], default="w",
                    help="what --offload-alpha moves: the W-stashes of microbatches whose weight gradients are "
                         "deferred (long-lived), the forward stashes (short-lived in a one-stage sequence), or both")
    ap.add_argument("--print-gemm", action="store_true",
                    help="with --only-gemm: print the leg's result as JSON, with per-shape times of this kernel and of the "
                         "vendor library on random and on zero operands")
    ap.add_argument("--gemm-shape", default=None, metavar="M,N,K",
                    help="with --only-gemm: time this one shape (forward layout) instead of the workload's four")
    ap.add_argument("--gemm-operands", choices=["random", "zeros"], default="random",
                    help="with --only-gemm: operand data of the replayed launches")
    ap.add_argument("--only-step", action="store_true",
                    help="run only the braided steps (warm-up + timed region) and print their time: under "
                         "rocprofv3 --kernel-trace --stats every kernel average is then a per-step figure")
    ap.add_argument("--only-gemm", action="store_true",
                    help="run only the dominant-kernel leg plus a 1 GiB device copy (counter calibration runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the TP all-reduce points are marked boundaries, "
              "no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.offload_alpha is not None:
        # The offload adds two copy streams to the three compute streams.  HIP maps a process's streams onto 4
        # hardware queues by default, so a fifth stream shares a queue with a compute stream, and a reload that
        # is enqueued ahead of time then sits behind every kernel already queued there.  Read at HIP start-up.
        if int(os.environ.get("GPU_MAX_HW_QUEUES", "4")) < 8:
            os.environ["GPU_MAX_HW_QUEUES"] = "8"

    import torch
    import paper_2510_27257_amd as stp
    from paper_2510_27257_amd import synth
    from paper_2510_27257_amd.binding import OP_B, OP_BW
    from paper_2510_27257_amd.stage import StageOnDevice, backward_ops, braid, forward_ops, weight_ops

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    fl = unit_flops(wl)
    total_flops = fl["F"] + fl["B"] + fl["W"]

    ctx = stp.Context(0)
    if args.gemm_shape:
        global GEMM_SHAPE_OVERRIDE
        GEMM_SHAPE_OVERRIDE = tuple(int(v) for v in args.gemm_shape.split(","))
    if args.only_gemm:
        ms, fl = gemm_leg(ctx, wl, max(10, args.steps), torch, stp, operands=args.gemm_operands)
        if args.print_gemm:
            line = {"avg_launch_ms": ms, "flops_per_launch": fl, "tflops": fl / (ms * 1e-3) / 1e12,
                    "operands": args.gemm_operands, "shapes_MNK": gemm_shapes(wl), "per_shape_ms": {}}
            for operands in ("random", "zeros"):
                for library in (False, True):
                    line["per_shape_ms"][("library_" if library else "this_kernel_") + operands] = gemm_leg(
                        ctx, wl, 20, torch, stp, operands=operands, library=library, per_shape=True)
            print(json.dumps(line))
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)          # plain copy of known size: 1 GiB read + 1 GiB written per launch
        torch.cuda.synchronize()
        ctx.close()
        return
    if args.stage:
        stage_bench(ctx, args, torch, stp, synth)
        ctx.close()
        return
    stg = StageOnDevice(ctx, [wl], n_mb=2, seed=0, tuned_tiles=not args.no_tuned_tiles)
    stg.load_inputs()
    sF, sB, sW = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    s0 = torch.cuda.current_stream()

    # prime: forward of microbatch 0 leaves the stash its backward needs
    ctx.braid_reset()
    ctx.braid_step(stg.stage, forward_ops(1, 0), s0, s0, s0)
    torch.cuda.synchronize()
    step_ops = braid(forward_ops(1, 1), backward_ops(1, 0, OP_BW))
    arr = (stp.Op * len(step_ops))(*step_ops)

    # ---- the timed region: K braided steps ------------------------------------------
    ms_braided = time_steps(lambda: ctx.braid_step(stg.stage, arr, sF, sB, sW), args.steps, args.warmup, torch)

    if args.only_step:
        print(json.dumps({"ms_per_step": ms_braided, "tflops": total_flops / (ms_braided * 1e-3) / 1e12,
                          "steps": args.steps, "warmup": args.warmup, "workload": wl.name}))
        torch.cuda.synchronize()
        ctx.close()
        return

    # ---- sustained shader clock while braided steps run (probe wave on a side stream) -------------
    probe_out = torch.zeros(2, dtype=torch.int64, device="cuda")
    s_probe = torch.cuda.Stream()
    n_probe = max(10, int(12.0 / ms_braided) + 4)
    for i in range(n_probe):
        ctx.braid_step(stg.stage, arr, sF, sB, sW)
        if i == 2:
            ctx.clock_probe(probe_out, 8.0, stream=s_probe)
    torch.cuda.synchronize()
    cyc, ticks = (int(v) for v in probe_out.tolist())
    wall_khz = ctx.wall_clock_khz()   # rate of the constant counter the probe reads beside the shader clock
    sustained_mhz = cyc / (ticks / wall_khz) / 1e3 if ticks else None
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count

    # ---- per-step makespans from HIP events (median over >= 20 steps) ----------------
    per_step = sorted(event_steps(ctx, stg.stage, arr, (sF, sB, sW), max(20, args.steps), torch))
    ms_median = per_step[len(per_step) // 2]

    # ---- the same op list on one stream, and the isolated units ----------------------
    ms_serial = time_steps(lambda: ctx.braid_step(stg.stage, arr, s0, s0, s0), args.steps, args.warmup, torch)
    f_ops = (stp.Op * 4)(*forward_ops(1, 1))
    b_ops = (stp.Op * 4)(*backward_ops(1, 0, OP_B))
    w_ops = (stp.Op * 2)(*weight_ops(1, 0))
    ms_F = time_steps(lambda: ctx.braid_step(stg.stage, f_ops, s0, s0, s0), args.steps, args.warmup, torch)
    ms_B = time_steps(lambda: ctx.braid_step(stg.stage, b_ops, s0, s0, s0), args.steps, args.warmup, torch)
    ms_W = time_steps(lambda: ctx.braid_step(stg.stage, w_ops, s0, s0, s0), args.steps, args.warmup, torch)

    T, h, a, f = wl.seq, wl.hidden, wl.attn_local, wl.ffn_local
    gemm_avg_ms, gemm_flops_per_launch = gemm_leg(ctx, wl, max(10, args.steps), torch, stp)
    achieved = gemm_flops_per_launch / (gemm_avg_ms * 1e-3) / 1e12

    hbm = hbm_leg(ctx, wl, torch, stp)

    result = {
        "metric": ("braided F/B/W TFLOP/s + MFMA util, 7B layer TP=8 shard, seq 6144, 1 GPU" if args.workload == "gpt7b_tp8"
                   else f"braided F/B/W TFLOP/s + MFMA util, workload {args.workload}, 1 GPU"),
        "value": total_flops / (ms_braided * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_braided,
        "ms_per_step_events": {"median": ms_median, "min": per_step[0], "max": per_step[-1], "n": len(per_step),
                               "tflops_at_median": total_flops / (ms_median * 1e-3) / 1e12,
                               "how": "HIP events after the end of every step on all three streams"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: hidden {h}, {wl.heads_local} local heads x {wl.head_dim}, ffn shard {f}, "
                               f"seq {T}, microbatch 1, tp {wl.tp}; step = F(mb1) braided with B+W(mb0), 1 layer",
                   "flops_per_step": total_flops,
                   "gemm_tile_hints": (f"{stg.n_tile_hints} measured tile preferences of paper_2510_27257_amd/tuned_tiles.json, "
                                       f"objective '{stg.tuned_objective}' (this block issued back to back)"
                                       if stg.tuned else "none (the library's own tile choice)")},
        "mfma_util_frac_of_bf16_peak": total_flops / (ms_braided * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
        "sustained_shader_clock_mhz": sustained_mhz,
        "sustained_shader_clock_source": "stp_clock_probe: one wave of one compute unit counting shader cycles for a 12 ms window while braided "
                                         "steps run; rocm-smi's chip-wide average over seconds is lower (about 1.95 GHz under this load: "
                                         "profiles/gemm_operand_data_and_clock.txt)",
        "mfma_util_frac_at_sustained_clock": (total_flops / (ms_braided * 1e-3) / 1e12 /
                                              (n_cu * 4096 * sustained_mhz * 1e6 / 1e12)) if sustained_mhz else None,
        "compute_units": n_cu,
        "units": {
            "F": {"ms": ms_F, "tflops": fl["F"] / (ms_F * 1e-3) / 1e12},
            "B": {"ms": ms_B, "tflops": fl["B"] / (ms_B * 1e-3) / 1e12},
            "W": {"ms": ms_W, "tflops": fl["W"] / (ms_W * 1e-3) / 1e12},
        },
        "braid": {"makespan_ms": ms_braided, "serialized_ms": ms_serial, "sum_isolated_ms": ms_F + ms_B + ms_W,
                  "makespan_over_sum_isolated": ms_braided / (ms_F + ms_B + ms_W)},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_dma_kernel<BM, BN, A k-contiguous, B row-contiguous, store> (forward layout; tile as picked per shape: 192x256 for all four when the GEMM has the GPU to itself)",
                     "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / BF16_MFMA_PEAK_TFLOPS, "avg_launch_ms": gemm_avg_ms,
                     "flops_per_launch": gemm_flops_per_launch,
                     "traffic": GEMM_FWD_TRAFFIC_BYTES if args.workload == "gpt7b_tp8" else None,
                     "traffic_source": GEMM_FWD_TRAFFIC_SOURCE if args.workload == "gpt7b_tp8" else None,
                     "algorithmic_bytes_per_launch": sum(2 * (M * K + K * N + M * N) for (M, N, K) in gemm_shapes(wl)) / 4,
                     "context": gemm_context(ctx, wl, max(10, args.steps), torch, stp)},
        "hbm_kernels": hbm,
        "attention_kernels": attention_leg(ctx, wl, torch, stp) if wl.dtype == "bf16" else None,
    }

    if not args.no_cpu_baseline:
        # the fp64 oracle, as it stands, on this machine's host cores: one full layer-microbatch, timed per unit kind
        result["cpu_baseline"] = cpu_baseline(wl, stg.w_host[0], fl, synth)
        tiny = synth.WORKLOADS["tiny"]
        result["cpu_baseline_tiny"] = cpu_baseline(tiny, synth.make_weights(tiny, 0), unit_flops(tiny), synth, reps=20)
    print(json.dumps(result))
    torch.cuda.synchronize()
    ctx.close()


if __name__ == "__main__":
    main()
