#!/usr/bin/env python3
"""Benchmark of the per-layer optimizer step on one MI355X.

A "step" is one pass of the whole hot path over one layer's tensors, all resident in HBM:
    gs_grad_sqnorm  (k bf16 gradient streams -> squared L2 norm, on device)
    gs_accum_adamw  (k-way accumulate + clip + AdamW on fp32 p/m/v + bf16 weight emit)
Default workload: one GPT-65B-shaped layer (h = 8192, 805 412 864 parameters, k = 16 bf16
micro-batch gradient buffers), synthetic seeded tensors.

Prints ONE JSON line.  `value` is parameters per second over the timed region (wall clock
between two device synchronisations).  `roofline` is for the dominant kernel
(gs_accum_adamw): algorithmic bytes (2k+26 per parameter) divided by its average duration
measured with HIP events on the launch stream (median and minimum beside it), against the
8 TB/s HBM peak; `roofline.achievable` holds what the same device gives simpler traffic and the
step's own mix of streams without arithmetic.  `cpu_baseline` times the CPU oracle on a bounded
sample of the same tensors on the host's cores, all of them and one.  With the default workload,
`other_workloads` adds short runs of the other configurations: the h = 1024 layer (cold caches:
rotating tensor sets), h = 4096, the GPT-30B-shaped layer, the split step of the GPT-175B-shaped
layer beside a GEMM, and the host-resident step (staged and in place).  `--workload NAME` runs
one of them in full instead.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
HEADLINE = "gpt65b_layer_h8192_k16"

# HBM bytes per gs_accum_adamw launch on the headline workload from rocprofv3 --pmc runs
# (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading on a plain copy kernel
# of known size); see profiles/.  None until measured for the workload being run.
MEASURED_TRAFFIC_BYTES = {"gpt65b_layer_h8192_k16": 46_712_867_821,    # profiles/gs_step_gpt65b_layer_h8192_k16.txt
                          "gpt_h4096_k8": 8_458_116_813}               # profiles/gs_step_gpt_h4096_k8.txt


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="headline workload only: skip the short runs of the other configurations")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the no-arithmetic stream-mix probe kernels")
    ap.add_argument("--k-sweep", action="store_true",
                    help="instead of the step benchmark: gs_accum_adamw and gs_grad_sqnorm on the workload's layer for "
                         "k = 1..32 gradient buffers (bytes per parameter 2k+26 and 2k), one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 2^28 floats (1 GiB in, 1 GiB out) three times before the "
                         "timed region, as the known-size reference for rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27, help="elements of the workload the oracle is timed on")
    ap.add_argument("--slots", type=int, default=3,
                    help="bounce slots of the tiered workload / staging slots of the streamed workload's copy-engine leg")
    ap.add_argument("--stream-cus", type=int, default=32,
                    help="compute units the host-resident step may use in the streamed and tiered workloads (0 = all)")
    ap.add_argument("--tier-dir", default=None, help="directory for the file tier's state files (default: the system temp dir)")
    ap.add_argument("--tier-direct", action="store_true",
                    help="open the file tier's state files with O_DIRECT (no page cache: the storage device's own rate)")
    return ap.parse_args()


def cpu_baseline(wl, p, m, v, grads, hp, sample: int):
    """Time the oracle (norm pass + fused step, as it stands) on the first `sample` elements of the
    workload's tensors: once split over the host's cores in disjoint ranges (the reported `value`),
    once on one thread over a quarter of that sample (`single_thread`)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    from oracle import gs_oracle as O
    from paper_2512_17570_amd import inputs as I

    sample = min(sample, wl.n)
    cores = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)
    cores = max(1, min(cores, os.cpu_count() or 1))
    h_p, h_m, h_v = (t[:sample].cpu().numpy().copy() for t in (p, m, v))
    h_g = [I.bf16_bits(g[:sample]).copy() for g in grads]
    h_w = np.zeros(sample, np.uint16)
    ohp = O.HParams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.max_grad_norm, hp.step)
    O.lib()

    def run(threads, count):
        bounds = [count * i // threads for i in range(threads + 1)]
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            S = sum(ex.map(lambda i: O.grad_sqnorm(h_g, bounds[i], bounds[i + 1]), range(threads)))
            c = O.clip_coef(S, hp.max_grad_norm)
            list(ex.map(lambda i: O.accum_adamw(h_p, h_m, h_v, h_w, h_g, ohp, c, bounds[i], bounds[i + 1]), range(threads)))
        return time.perf_counter() - t0

    dt = run(cores, sample)
    single = max(1, sample // 4)
    dt1 = run(1, single)
    try:
        model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except Exception:
        model = "unknown"
    return {"value": sample / dt, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample} of {wl.n} parameters of the same tensors, norm pass + fused step, "
                      f"{cores} threads over disjoint ranges, {dt:.2f} s wall",
            "single_thread": {"value": single / dt1, "unit": "params/s", "cores": 1,
                              "sample": f"first {single} parameters, norm pass + fused step, one thread, {dt1:.2f} s wall"},
            "host_cpu": model, "host_logical_cpus": os.cpu_count()}


def _hp_of(gs, wl, i=0):
    return gs.HParams(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.max_grad_norm, wl.step + i)


def _base_record(wl, props, value, steps, warmup, ms_per_step, extra_cfg=None):
    cfg = {"workload": wl.name, "h": wl.h, "layers": wl.layers, "n_params": wl.n, "k_grad_buffers": wl.k,
           "grad_dtype": "bf16", "state_dtype": "f32", "clip_max_norm": wl.max_grad_norm,
           "device": props.name, "compute_units": props.multi_processor_count, "hbm_bytes": props.total_memory}
    cfg.update(extra_cfg or {})
    return {"metric": "params/s, fused grad-norm + accumulate + AdamW step", "value": value, "unit": "params/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": cfg}


NOTES = []       # anything the run wants the reader of the JSON line to know (printed as "notes" when non-empty)


def runs_beside(torch, a, b, big=None):
    """True if work on stream b overtakes a burst already running on stream a (different hardware queues)."""
    own = big is None
    if own:
        big = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
    small = torch.zeros(1 << 10, dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    e_long, e_short = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(a):
        for _ in range(8):
            big.add_(1.0)
        e_long.record(a)
    with torch.cuda.stream(b):
        small.add_(1.0)
        e_short.record(b)
    torch.cuda.synchronize()
    return e_short.elapsed_time(e_long) >= 0.5


def concurrent_streams(torch, count=2, tries=24):
    """`count` torch streams that the runtime really runs side by side.  HIP multiplexes a process's
    streams onto a few hardware queues (4 here), and two streams that land on one queue run their
    work in turn, which would turn every "beside" measurement below into a serial one.  A candidate
    is accepted when a tiny kernel launched on it AFTER a few-millisecond burst on each stream
    already chosen finishes BEFORE that burst does."""
    big = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
    small = torch.zeros(1 << 10, dtype=torch.float32, device="cuda:0")
    big.zero_()
    chosen = [torch.cuda.Stream()]
    for _ in range(tries):
        if len(chosen) == count:
            break
        cand = torch.cuda.Stream()
        if any(cand.cuda_stream == c.cuda_stream for c in chosen):
            continue
        ok = True
        for c in chosen:
            torch.cuda.synchronize()
            e_long, e_short = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(c):
                for _ in range(8):
                    big.add_(1.0)
                e_long.record(c)
            with torch.cuda.stream(cand):
                small.add_(1.0)
                e_short.record(cand)
            torch.cuda.synchronize()
            if e_short.elapsed_time(e_long) < 0.5:      # the tiny kernel did not overtake the burst
                ok = False
                break
        if ok:
            chosen.append(cand)
    del big, small
    while len(chosen) < count:
        # no candidate passed: carry on with unverified streams and say so in the record
        chosen.append(torch.cuda.Stream())
        NOTES.append("concurrent_streams: no stream pair was seen to run side by side; a 'beside' figure in this record "
                     "may be a serial one")
    return chosen


def _layer_sequence(args, wl, gs, torch, dev, tokens, ga, gb, gc, sa, step_args, t_def, cus):
    p, m, v, w, grads, s_pt, n, sq = step_args
    # A sequence of layers (Sec. 4.4: a layer's deferred update only has to be finished before that
    # layer's forward of the next iteration): the forward of layer i (its four bf16 GEMMs for
    # `tokens` tokens) waits for the event of layer i's deferred step; the deferred steps run in
    # layer order on their own stream, so step i+1 overlaps forward i.  Every "layer" reuses the
    # same state and weight tensors: this times the schedule, not the arithmetic.
    seq_layers = 6
    wq = torch.randn(wl.h, 3 * wl.h, dtype=torch.bfloat16, device=dev)
    wo = gb
    w1 = torch.randn(wl.h, 4 * wl.h, dtype=torch.bfloat16, device=dev)
    w2 = torch.randn(4 * wl.h, wl.h, dtype=torch.bfloat16, device=dev)
    o_q = torch.empty(tokens, 3 * wl.h, dtype=torch.bfloat16, device=dev)
    o_1 = torch.empty(tokens, 4 * wl.h, dtype=torch.bfloat16, device=dev)

    def forward_layer():
        torch.matmul(ga, wq, out=o_q)
        torch.matmul(ga, wo, out=gc)
        torch.matmul(ga, w1, out=o_1)
        torch.matmul(o_1, w2, out=gc)

    def sequence(num_cus, overlap, reps):
        """One iteration = the deferred steps of all layers handed to a gs_defer_ctx (its own stream, on a
        budget of num_cus compute units if > 0) and the forwards on `sa`, each behind its layer's deadline
        (overlap) or behind the last layer's (serial)."""
        # a context whose stream really runs beside the forward's stream (see concurrent_streams)
        rejected, ctx = [], None
        for _ in range(8):
            ctx = gs.gs_defer_ctx_create(seq_layers, num_cus)
            if runs_beside(torch, sa, torch.cuda.ExternalStream(gs.gs_defer_ctx_stream(ctx))):
                break
            rejected.append(ctx)
        for r in rejected:
            gs.gs_defer_ctx_destroy(r)
        hp = _hp_of(gs, wl)

        def once():
            for i in range(seq_layers):
                gs.gs_defer_layer_step(ctx, i, p, m, v, w, grads, s_pt, n, hp, sq, producer_stream=sa)
            with torch.cuda.stream(sa):
                if not overlap:
                    gs.gs_defer_wait_layer(ctx, seq_layers - 1, sa)
                for i in range(seq_layers):
                    if overlap:
                        gs.gs_defer_wait_layer(ctx, i, sa)
                    forward_layer()
            # the next iteration's steps follow this iteration's forward (producer_stream = sa)
        once()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            once()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps * 1e3
        gs.gs_defer_ctx_destroy(ctx)
        return dt

    with torch.cuda.stream(sa):
        for _ in range(2):
            forward_layer()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(sa):
        e0.record(sa)
        for _ in range(seq_layers):
            forward_layer()
        e1.record(sa)
    torch.cuda.synchronize()
    t_fwd_layer = e0.elapsed_time(e1) / seq_layers
    seq_reps = max(2, args.steps // 4)
    seq = {"layers": seq_layers, "forward_ms_per_layer_alone": t_fwd_layer,
           "forward_TFLOPs_alone": 2.0 * tokens * wl.h * 12 * wl.h / (t_fwd_layer * 1e-3) / 1e12,
           "deferred_ms_per_layer_alone": t_def,
           "serial_ms": sequence(0, False, seq_reps),
           "overlapped_all_cus_ms": sequence(0, True, seq_reps)}
    for ncu in (cus // 4, cus // 2):
        seq[f"overlapped_{ncu}_cus_ms"] = sequence(ncu, True, seq_reps)
    seq["bound_ms"] = t_def + seq_layers * t_fwd_layer      # first step exposed, everything else hidden
    seq["note"] = ("gs_defer_ctx: forward of layer i waits for layer i's deadline (gs_defer_wait_layer); steps run in layer "
                   "order on the context's stream. "
                   "bound = one exposed deferred step + the forwards at their solo speed")

    return seq


def bench_split(args, wl, brief=False):
    """Split step (delay ratio alpha, Sec. 4.4 of the paper): the immediate part of the range is
    updated right away, the deferred part on a second stream while a bf16 GEMM standing in for the
    next iteration's forward runs on the first.  Reports the step's and the GEMM's slowdown under
    contention.  Timing only; split == full is checked bit for bit by the GPU tests."""
    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    dev = "cuda:0"
    props = torch.cuda.get_device_properties(0)
    n, k = wl.n, wl.k
    s_pt = int(wl.extra["immediate_frac"] * n)
    p, m, v, grads = I.make_workload_tensors(wl, dev)
    w = torch.zeros(n, dtype=torch.bfloat16, device=dev)
    sq = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
    tokens = wl.extra["gemm_tokens"]
    ga = torch.randn(tokens, wl.h, dtype=torch.bfloat16, device=dev)
    gb = torch.randn(wl.h, wl.h, dtype=torch.bfloat16, device=dev)
    gc = torch.empty(tokens, wl.h, dtype=torch.bfloat16, device=dev)
    sa, sb = concurrent_streams(torch, 2)
    hp = _hp_of(gs, wl)
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    torch.cuda.synchronize()

    def timed(fn, stream, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            e0.record(stream)
            for _ in range(reps):
                fn(stream)
            e1.record(stream)
        return e0, e1

    def full(st):
        gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq, stream=st)

    def immediate(st):
        gs.gs_accum_adamw(p, m, v, w, grads, 0, s_pt, hp, sq, stream=st)

    def deferred(st):
        gs.gs_accum_adamw(p, m, v, w, grads, s_pt, n, hp, sq, stream=st)

    def gemm(st):
        torch.matmul(ga, gb, out=gc)

    def alone(fn, stream, reps):
        for _ in range(args.warmup):
            with torch.cuda.stream(stream):
                fn(stream)
        torch.cuda.synchronize()
        e0, e1 = timed(fn, stream, reps)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # split == full, bit for bit, on the tensors being timed: the full step on the states, the immediate and
    # the deferred part (two streams) on a copy of them, same hyper-parameters and norm
    p2, m2, v2, w2 = p.clone(), m.clone(), v.clone(), torch.zeros_like(w)
    torch.cuda.synchronize()
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)
    torch.cuda.synchronize()
    gs.gs_accum_adamw(p2, m2, v2, w2, grads, 0, s_pt, hp, sq, stream=sa)
    gs.gs_accum_adamw(p2, m2, v2, w2, grads, s_pt, n, hp, sq, stream=sb)
    torch.cuda.synchronize()
    split_equals_full = all(torch.equal(a.view(torch.int32 if a.dtype == torch.float32 else torch.int16),
                                        b.view(torch.int32 if b.dtype == torch.float32 else torch.int16))
                            for a, b in ((p, p2), (m, m2), (v, v2), (w, w2)))
    del p2, m2, v2, w2

    t_full = alone(full, sb, args.steps)
    t_imm = alone(immediate, sb, args.steps)
    t_def = alone(deferred, sb, args.steps)
    t_gemm = alone(gemm, sa, 4 * args.steps)
    reps_gemm = max(1, int(round(t_def / t_gemm)))     # GEMMs that cover one deferred step
    # concurrent: each iteration = one deferred step on sb || reps_gemm GEMMs on sa
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pairs = []
    for _ in range(args.steps):
        eg = timed(gemm, sa, reps_gemm)
        ed = timed(deferred, sb, 1)
        pairs.append((eg, ed))
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps * 1e3
    t_gemm_c = sum(a.elapsed_time(b) for (a, b), _ in pairs) / args.steps / reps_gemm
    t_def_c = sum(a.elapsed_time(b) for _, (a, b) in pairs) / args.steps
    # the same with the deferred part on a stream confined to half of the compute units
    budget = {}
    cus = props.multi_processor_count
    for ncu in (() if brief else (cus // 2, (3 * cus) // 4)):
        raw = gs.gs_cu_stream_create(ncu)
        sc = torch.cuda.ExternalStream(raw)
        t_def_b = alone(deferred, sc, args.steps)
        reps_b = reps_gemm
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pairs_b = []
        for _ in range(args.steps):
            eg = timed(gemm, sa, reps_b)
            ed = timed(deferred, sc, 1)
            pairs_b.append((eg, ed))
        torch.cuda.synchronize()
        wall_b = (time.perf_counter() - t0) / args.steps * 1e3
        budget[str(ncu)] = {
            "deferred_alone_ms": t_def_b,
            "deferred_concurrent_ms": sum(a.elapsed_time(b) for _, (a, b) in pairs_b) / args.steps,
            "gemm_concurrent_ms": sum(a.elapsed_time(b) for (a, b), _ in pairs_b) / args.steps / reps_b,
            "concurrent_wall_ms_per_iter": wall_b}
        budget[str(ncu)]["gemm_slowdown"] = budget[str(ncu)]["gemm_concurrent_ms"] / t_gemm
        del sc
        gs.gs_cu_stream_destroy(raw)
    seq = None
    if not brief:
        seq = _layer_sequence(args, wl, gs, torch, dev, tokens, ga, gb, gc, sa, (p, m, v, w, grads, s_pt, n, sq), t_def, cus)

    bpp = 2 * k + 26
    rec = _base_record(wl, props, n / ((t_imm + t_def) * 1e-3), args.steps, args.warmup, t_imm + t_def,
                       {"split_point": s_pt, "immediate_frac": wl.extra["immediate_frac"],
                        "gemm": f"bf16 {tokens}x{wl.h} @ {wl.h}x{wl.h}", "gemms_per_deferred_step": reps_gemm})
    rec["roofline"] = {"bound": "hbm", "kernel": "gs_accum_adamw (full range)", "achieved": n * bpp / (t_full * 1e-3) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": n * bpp / (t_full * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "traffic": None, "algorithmic_bytes_per_launch": n * bpp, "avg_launch_ms": t_full}
    gemm_flop = 2.0 * tokens * wl.h * wl.h
    rec["split"] = {
        "split_equals_full_bitwise": bool(split_equals_full),
        "full_ms": t_full, "immediate_ms": t_imm, "deferred_alone_ms": t_def,
        "deferred_alone_GBps": (n - s_pt) * bpp / (t_def * 1e-3) / 1e9,
        "gemm_alone_ms": t_gemm, "gemm_alone_TFLOPs": gemm_flop / (t_gemm * 1e-3) / 1e12,
        "deferred_concurrent_ms": t_def_c, "gemm_concurrent_ms": t_gemm_c,
        "deferred_slowdown": t_def_c / t_def, "gemm_slowdown": t_gemm_c / t_gemm,
        "concurrent_wall_ms_per_iter": wall, "serial_ms_per_iter": t_def + reps_gemm * t_gemm,
        "deferred_on_cu_budget_stream": budget,
        "layer_sequence": seq,
    }
    rec["cpu_baseline"] = None
    return rec


def bench_streamed(args, wl, brief=False):
    """Host-resident step (Sec. 2.2 chunk loop / Sec. 4.3 pipeline of the paper, with host<->GPU
    PCIe as the slow link): fp32 p/m/v of all layers live in pinned host memory and are stepped in
    2^26-element chunks, upload | kernel | download overlapped on three streams (12 B up + 12 B down
    per parameter).  Reports params/s against the one-directional pinned-copy rate of this host,
    measured after the timed region with raw hipMemcpyAsync, and beside it the same passes with the
    kernel in place on the host arrays (one stream limited to --stream-cus compute units)."""
    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    dev = "cuda:0"
    props = torch.cuda.get_device_properties(0)
    chunk = wl.extra["chunk_elems"]
    layers, nl, k = wl.layers, I.layer_numel(wl.h), wl.k
    steps, warmup = (min(args.steps, 3), 1) if brief else (args.steps, args.warmup)
    if brief:
        layers = min(layers, 2)
    # pin as many layers as the host allows
    bufs = None
    while layers > 0:
        bufs = gs.pinned_f32_set(layers * nl, 3)
        if bufs is not None:
            break
        layers -= 1
    if layers == 0:
        print("bench.py: cannot pin host memory for even one layer", file=sys.stderr)
        sys.exit(1)
    n = layers * nl
    (hp_t, hp_p), (hm_t, hm_p), (hv_t, hv_p) = bufs
    grads_l, w_l = [], []
    for L in range(layers):
        pd, md, vd = I.make_states(nl, wl.seed + L, dev)
        for dst, src in ((hp_t, pd), (hm_t, md), (hv_t, vd)):
            dst[L * nl:(L + 1) * nl].copy_(src)
        del pd, md, vd
        grads_l.append(I.make_grads(nl, k, wl.grad_sigma, wl.seed + L, dev))
        w_l.append(torch.zeros(nl, dtype=torch.bfloat16, device=dev))
    sq = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
    for L in range(layers):                      # global norm over all layers
        gs.gs_grad_sqnorm(grads_l[L], 0, nl, sq, ws, accumulate=(L > 0))
    torch.cuda.synchronize()

    cur = torch.cuda.current_stream()

    def timed_passes(ctx):
        def one_pass(i):
            hp = _hp_of(gs, wl, i)
            for L in range(layers):
                o = L * nl * 4
                gs.gs_stream_layer_step(ctx, hp_p + o, hm_p + o, hv_p + o, w_l[L], grads_l[L], nl, hp, sq,
                                        producer_stream=cur)
            gs.gs_stream_ctx_sync(ctx)
        for i in range(warmup):
            one_pass(i)
        t0 = time.perf_counter()
        for i in range(steps):
            one_pass(warmup + i)
        return (time.perf_counter() - t0) / steps

    # the configuration as named: 2^26-element chunks, upload | kernel in an HBM slot | download
    ctx = gs.gs_stream_ctx_create(chunk, args.slots)
    copies_overlap = gs.gs_stream_ctx_copies_overlap(ctx)
    per = timed_passes(ctx)
    gs.gs_stream_ctx_destroy(ctx)
    # the same passes with the kernel in place on the pinned host arrays: reported beside `value`
    ctx = gs.gs_stream_ctx_create_inplace(args.stream_cus)
    per_inplace = timed_passes(ctx)
    gs.gs_stream_ctx_destroy(ctx)

    # the link's ceilings, measured afterwards: raw pinned hipMemcpyAsync of 2^26-element pieces,
    # one way at a time and both ways at once
    import ctypes
    hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))
    hip.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    hip.hipMemcpyAsync.restype = ctypes.c_int
    up, dn = concurrent_streams(torch, 2)          # two streams on different hardware queues
    stage = [torch.empty(chunk, dtype=torch.float32, device=dev) for _ in range(2)]
    stage[1].zero_()

    def copy_pass(nchunks, h2d, d2h):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in range(nchunks):
            lo = ((c * chunk) % max(1, n - chunk)) * 4
            if h2d:
                r = hip.hipMemcpyAsync(stage[0].data_ptr(), hp_p + lo, chunk * 4, 1, up.cuda_stream)
                assert r == 0, r
            if d2h:
                r = hip.hipMemcpyAsync(hm_p + lo, stage[1].data_ptr(), chunk * 4, 2, dn.cuda_stream)
                assert r == 0, r
        torch.cuda.synchronize()
        return nchunks * chunk * 4 / (time.perf_counter() - t0) / 1e9

    copy_pass(8, True, True)                      # warm the copy engines and both streams
    h2d_only_gbs = copy_pass(16 if brief else 32, True, False)
    d2h_only_gbs = copy_pass(16 if brief else 32, False, True)
    duplex_dir_gbs = copy_pass(24 if brief else 48, True, True)
    del stage

    rec = _base_record(wl, props, n / per, steps, warmup, per * 1e3,
                       {"layers": layers, "layers_in_workload": wl.layers, "n_params": n, "chunk_elems": chunk,
                        "slots": args.slots,
                        "host_pinned_bytes": 12 * n, "device_staging_bytes": args.slots * 3 * (chunk + 64) * 4,
                        "copies_overlap_check": copies_overlap})
    pcie_dir = 12 * n / per / 1e9
    link = min(h2d_only_gbs, d2h_only_gbs)
    rec["roofline"] = {"bound": "pcie", "kernel": "gs_stream_layer_step, staged (H2D 12 B + D2H 12 B per parameter)",
                       "achieved": pcie_dir, "peak": link, "unit": "GB/s per direction",
                       "frac": pcie_dir / link, "traffic": None,
                       "peak_source": "measured on this host after the timed region: one-directional pinned hipMemcpyAsync "
                                      "(the slower of H2D and D2H); a full-duplex link would sustain it both ways",
                       "h2d_only_GBps": h2d_only_gbs, "d2h_only_GBps": d2h_only_gbs,
                       "duplex_copy_probe_GBps_per_direction": duplex_dir_gbs,
                       "params_per_s_bound": link * 1e9 / 12}
    rec["in_place"] = {
        "params_per_s": n / per_inplace, "ms_per_step": per_inplace * 1e3,
        "GBps_per_direction": 12 * n / per_inplace / 1e9, "frac_of_link": 12 * n / per_inplace / 1e9 / link,
        "stream_cus": args.stream_cus, "device_staging_bytes": 0,
        "note": "gs_stream_ctx_create_inplace: the step kernel runs on the pinned host arrays (12 B read + 12 B written "
                "over the link per parameter), one stream limited to stream_cus compute units, no copies; same results "
                "bit for bit; its rate does not depend on the runtime's copy path or on hardware-queue assignment"}
    rec["cpu_baseline"] = None
    for t, ptr in bufs:
        gs.gs_pinned_free(ptr)
    return rec


def bench_tiered(args, wl):
    """Three-tier step (Sec. 4.3 pipeline with the SSD leg, Sec. 4.5 storage ratio): a share x of
    every layer's fp32 p/m/v lives in pinned host memory, the rest in files under --tier-dir; file
    chunks are read into pinned bounce slots, go through the host<->HBM pipeline and are written
    back by a writer thread.  Reports params/s and the file tier's GB/s per direction against raw
    pread/pwrite of the same files measured here (three threads, like the pipeline's)."""
    import shutil
    import tempfile
    import threading

    import numpy as np
    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    dev = "cuda:0"
    props = torch.cuda.get_device_properties(0)
    chunk, x = wl.extra["chunk_elems"], wl.extra["host_share"]
    layers, nl, k = wl.layers, I.layer_numel(wl.h), wl.k
    n_host = int(round(x * nl))
    n_file = nl - n_host
    root = tempfile.mkdtemp(prefix="gs_tier_", dir=args.tier_dir)
    free = shutil.disk_usage(root).free
    while layers > 1 and layers * n_file * 12 > 0.8 * free:
        layers -= 1
    hosts, fds, grads_l, w_l = [], [], [], []
    try:
        for L in range(layers):
            pd, md, vd = I.make_states(nl, wl.seed + L, dev)
            bufs = gs.pinned_f32_set(max(n_host, 1), 3)
            if bufs is None:
                print("bench.py: cannot pin the host share", file=sys.stderr)
                sys.exit(1)
            hosts.append(bufs)
            lf = []
            for name, (t, _), src in zip("pmv", bufs, (pd, md, vd)):
                t[:n_host].copy_(src[:n_host])
                path = os.path.join(root, f"L{L}_{name}.bin")
                src[n_host:].cpu().numpy().tofile(path)
                lf.append(os.open(path, os.O_RDWR | (os.O_DIRECT if args.tier_direct else 0)))
            fds.append(lf)
            del pd, md, vd
            grads_l.append(I.make_grads(nl, k, wl.grad_sigma, wl.seed + L, dev))
            w_l.append(torch.zeros(nl, dtype=torch.bfloat16, device=dev))
        sq = torch.zeros(1, dtype=torch.float64, device=dev)
        ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
        for L in range(layers):
            gs.gs_grad_sqnorm(grads_l[L], 0, nl, sq, ws, accumulate=(L > 0))
        torch.cuda.synchronize()

        # raw file ceilings: p/m/v of every layer read (then written) chunk by chunk by three threads
        import mmap
        scratch = [mmap.mmap(-1, chunk * 4) for _ in range(3)]      # page-aligned, as O_DIRECT needs

        def sweep(write):
            def worker(a):
                buf = memoryview(scratch[a])
                for L in range(layers):
                    for off in range(0, n_file * 4, chunk * 4):
                        ln = min(chunk * 4, n_file * 4 - off)
                        if write:
                            os.pwrite(fds[L][a], buf[:ln], off)
                        else:
                            os.preadv(fds[L][a], [buf[:ln]], off)
            ths = [threading.Thread(target=worker, args=(a,)) for a in range(3)]
            t0 = time.perf_counter()
            for t in ths:
                t.start()
            for t in ths:
                t.join()
            return layers * n_file * 12 / (time.perf_counter() - t0) / 1e9

        print(f"[tiered] {layers} layers staged under {root}, {layers * n_file * 12 / 1e9:.1f} GB in files", file=sys.stderr, flush=True)
        if not args.tier_direct:
            sweep(False)                          # warm the page cache
        read_gbs = sweep(False)
        print(f"[tiered] raw pread {read_gbs:.2f} GB/s", file=sys.stderr, flush=True)
        write_gbs = None
        if n_file:
            # write back what was just read, so the files keep their contents
            def rw_worker(a, out):
                buf = memoryview(scratch[a])
                t_w = 0.0
                for L in range(layers):
                    for off in range(0, n_file * 4, chunk * 4):
                        ln = min(chunk * 4, n_file * 4 - off)
                        os.preadv(fds[L][a], [buf[:ln]], off)
                        t0 = time.perf_counter()
                        os.pwrite(fds[L][a], buf[:ln], off)
                        t_w += time.perf_counter() - t0
                out[a] = t_w
            out = [0.0] * 3
            ths = [threading.Thread(target=rw_worker, args=(a, out)) for a in range(3)]
            for t in ths:
                t.start()
            for t in ths:
                t.join()
            write_gbs = layers * n_file * 12 / max(out) / 1e9

        ctx = gs.gs_tier_ctx_create(chunk, args.slots, args.stream_cus)
        cur = torch.cuda.current_stream()

        issue_s = []         # time the caller spends inside the (queueing) calls of one pass

        def one_pass(i):
            hp = _hp_of(gs, wl, i)
            t_issue = time.perf_counter()
            for L in range(layers):
                (_, pp), (_, pm), (_, pv) = hosts[L]
                gs.gs_tier_layer_step(ctx, pp, pm, pv, n_host, fds[L], (0, 0, 0), w_l[L], grads_l[L], nl, hp, sq,
                                      producer_stream=cur)
            issue_s.append(time.perf_counter() - t_issue)
            gs.gs_tier_ctx_sync(ctx)

        print(f"[tiered] raw pwrite {write_gbs} GB/s; timing", file=sys.stderr, flush=True)
        for i in range(args.warmup):
            one_pass(i)
        t0 = time.perf_counter()
        for i in range(args.steps):
            one_pass(args.warmup + i)
            print(f"[tiered] pass {i + 1}/{args.steps} at {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
        elapsed = time.perf_counter() - t0
        gs.gs_tier_ctx_destroy(ctx)
        per = elapsed / args.steps
        n = layers * nl

        # both directions at once on the same device (after the timed run: this overwrites the last
        # layer's files): three threads read the first layer's files while three write the last layer's
        duplex_gbs = None
        if n_file:
            wbuf = [mmap.mmap(-1, chunk * 4) for _ in range(3)]

            def dworker(a, write):
                buf = memoryview(wbuf[a] if write else scratch[a])
                L = layers - 1 if write else 0
                for off in range(0, n_file * 4, chunk * 4):
                    ln = min(chunk * 4, n_file * 4 - off)
                    if write:
                        os.pwrite(fds[L][a], buf[:ln], off)
                    else:
                        os.preadv(fds[L][a], [buf[:ln]], off)
            ths = [threading.Thread(target=dworker, args=(a, wr)) for a in range(3) for wr in (False, True)]
            t0 = time.perf_counter()
            for t in ths:
                t.start()
            for t in ths:
                t.join()
            duplex_gbs = n_file * 12 / (time.perf_counter() - t0) / 1e9
        rec = _base_record(wl, props, n / per, args.steps, args.warmup, per * 1e3,
                           {"layers": layers, "n_params": n, "chunk_elems": chunk, "slots": args.slots,
                            "host_share_x": x, "file_bytes": layers * n_file * 12, "host_pinned_bytes": layers * n_host * 12,
                            "tier_dir": os.path.dirname(root), "o_direct": bool(args.tier_direct), "stream_cus": args.stream_cus,
                            "tier_dir_fs_free_bytes": free,
                            "caller_blocked_ms_per_pass": 1e3 * sum(issue_s[args.warmup:]) / max(1, args.steps)})
        file_dir = layers * n_file * 12 / per / 1e9
        # the pipeline reads and writes at once, so the both-at-once probe is the ceiling it is held against
        peak = duplex_gbs if duplex_gbs else (min(read_gbs, write_gbs) if write_gbs else read_gbs)
        rec["roofline"] = {"bound": "file", "kernel": "gs_tier_layer_step (file share: 12 B read + 12 B written per parameter)",
                           "achieved": file_dir, "peak": peak, "unit": "GB/s per direction", "frac": file_dir / peak,
                           "traffic": None,
                           "peak_source": "measured here on the same files: three threads reading one layer's files while three "
                                          "write another's, chunk-sized requests "
                                          + ("with O_DIRECT, as in the timed run" if args.tier_direct else
                                             "(page cache included, as in the timed run; no fsync)"),
                           "pread_GBps": read_gbs, "pwrite_GBps": write_gbs,
                           "duplex_probe_GBps_per_direction": duplex_gbs,
                           "pcie_GBps_per_direction": 12 * n / per / 1e9}
        rec["cpu_baseline"] = None
        return rec
    finally:
        for lf in fds:
            for fd in lf:
                os.close(fd)
        shutil.rmtree(root, ignore_errors=True)
        for bufs in hosts:
            for _, ptr in bufs:
                gs.gs_pinned_free(ptr)


CACHE_BYTES = 256 << 20        # last-level (memory-side) cache of the device; L2 is 8 x 4 MB on top
COLD_SETS = 8


def _stats(ms):
    """Mean, median and minimum of a list of per-launch durations (ms)."""
    xs = sorted(ms)
    nn = len(xs)
    med = xs[nn // 2] if nn % 2 else 0.5 * (xs[nn // 2 - 1] + xs[nn // 2])
    return {"avg_ms": sum(xs) / nn, "median_ms": med, "min_ms": xs[0]}


def _kernel_entry(ms, bytes_per_param, n):
    st = _stats(ms)
    nbytes = n * bytes_per_param
    st.update({"bytes_per_param": bytes_per_param, "GBps": nbytes / (st["avg_ms"] * 1e-3) / 1e9,
               "frac": nbytes / (st["avg_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "GBps_median": nbytes / (st["median_ms"] * 1e-3) / 1e9, "GBps_best": nbytes / (st["min_ms"] * 1e-3) / 1e9})
    return st


def same_mix_ceiling(torch, grads, p, m, v, w, n, k, reps, block):
    """What this device gives the fused step's own mix of streams (k bf16 + 3 fp32 in, 3 fp32 + 1 bf16
    out) when no arithmetic is attached: the probe kernels of probe/gs_mixprobe.hip, out of place
    into scratch outputs.  (a) the step kernel's shape; (b) the same tile with all loads in flight;
    (c) the read half and the write half as two kernels running at once on two streams."""
    from paper_2512_17570_amd import mixprobe as MP

    dev = p.device
    n4 = n - n % 4
    po, mo, vo = torch.empty_like(p), torch.empty_like(m), torch.empty_like(v)
    wo = torch.empty_like(w)
    sink = torch.zeros(16, dtype=torch.int32, device=dev)
    s1, s2 = concurrent_streams(torch, 2)
    total = n4 * (2 * k + 26)

    def timed_one(mode, blk):
        def go():
            MP.launch(mode, blk, p, m, v, po, mo, vo, wo, grads, n4, sink, s1)
        go()
        s1.synchronize()
        out = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s1)
            go()
            e1.record(s1)
            s1.synchronize()
            out.append(e0.elapsed_time(e1))
        return out

    fused = timed_one(MP.FUSED_SHALLOW, block)
    deep = timed_one(MP.FUSED_ALL_IN_FLIGHT, 256)
    rd = timed_one(MP.READ_HALF, block)
    wr = timed_one(MP.WRITE_HALF, block)
    # both halves at once: the read kernel on s1, the write kernel on s2, started together
    pair = []
    for it in range(reps + 1):
        torch.cuda.synchronize()
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(s1)
        s2.wait_event(e0)
        MP.launch(MP.READ_HALF, block, p, m, v, po, mo, vo, wo, grads, n4, sink, s1)
        MP.launch(MP.WRITE_HALF, block, p, m, v, po, mo, vo, wo, grads, n4, sink, s2)
        e1.record(s1)
        e2.record(s2)
        torch.cuda.synchronize()
        if it:
            pair.append(max(e0.elapsed_time(e1), e0.elapsed_time(e2)))
    del po, mo, vo, wo

    def gbs(ms):
        return total / (_stats(ms)["avg_ms"] * 1e-3) / 1e9
    r_ms, w_ms = _stats(rd)["avg_ms"], _stats(wr)["avg_ms"]
    res = {"same_mix_step_shape_GBps": gbs(fused), "same_mix_all_loads_in_flight_GBps": gbs(deep),
           "same_mix_read_kernel_beside_write_kernel_GBps": gbs(pair),
           "read_half_alone_GBps": n4 * (2 * k + 12) / (r_ms * 1e-3) / 1e9,
           "write_half_alone_GBps": n4 * 14 / (w_ms * 1e-3) / 1e9,
           "read_then_write_serial_GBps": total / ((r_ms + w_ms) * 1e-3) / 1e9}
    res["same_mix_ceiling_GBps"] = max(res["same_mix_step_shape_GBps"], res["same_mix_all_loads_in_flight_GBps"])
    return res


def bench_resident(args, wl, full=True):
    """One layer resident in HBM: norm pass + fused step, timed per launch with events.  full: also the
    widened variants (staged two-pass, accumulate-as-you-go, speculative), the achievable ceilings
    and the CPU baseline (the headline record); otherwise the two kernels only."""
    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    dev = "cuda:0"
    props = torch.cuda.get_device_properties(0)
    n, k = wl.n, wl.k
    working_set = n * (12 + 2 + 2 * k)
    # A working set near the size of the last-level cache would be timed warm on one tensor set, so
    # small workloads rotate over independent sets (one per iteration, round robin): by the time a
    # set comes round again, COLD_SETS-1 others have streamed through the caches.
    nsets = COLD_SETS if working_set < 4 * CACHE_BYTES else 1

    t_gen = time.perf_counter()
    sets = []
    for r in range(nsets):
        p, m, v = I.make_states(n, wl.seed + 1000 * r, dev)
        grads = I.make_grads(n, k, wl.grad_sigma, wl.seed + 1000 * r, dev, wl.outlier_frac, wl.outlier_scale)
        sets.append((p, m, v, torch.zeros(n, dtype=torch.bfloat16, device=dev), grads))
    sq = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    p, m, v, w, grads = sets[0]

    def hp_at(i):
        return gs.HParams(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.max_grad_norm, wl.step + i)

    cpu = None
    if full and not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, p, m, v, grads, hp_at(0), args.cpu_sample)

    def one_step(i, evs=None, which=None):
        sp, sm, sv, sw, sg = sets[(i if which is None else which) % nsets]
        if evs:
            evs[0].record()
        gs.gs_grad_sqnorm(sg, 0, n, sq, ws)
        if evs:
            evs[1].record()
        gs.gs_accum_adamw(sp, sm, sv, sw, sg, 0, n, hp_at(i), sq)
        if evs:
            evs[2].record()

    if full and args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    warm = max(args.warmup, nsets if nsets > 1 else 0)      # every set is touched once before timing
    for i in range(warm):
        one_step(i)
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(warm + i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    norm_l = [e[0].elapsed_time(e[1]) for e in events]
    step_l = [e[1].elapsed_time(e[2]) for e in events]
    both_l = [e[0].elapsed_time(e[2]) for e in events]
    k_step = _kernel_entry(step_l, 2 * k + 26, n)
    k_norm = _kernel_entry(norm_l, 2 * k, n)

    warm_ref = None
    if nsets > 1:
        # the same on ONE tensor set, i.e. with whatever the caches keep from the previous iteration
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        for i in range(3):
            one_step(i, which=0)
        torch.cuda.synchronize()
        for i in range(args.steps):
            one_step(i, ev[i], which=0)
        torch.cuda.synchronize()
        warm_ref = {"gs_accum_adamw": _kernel_entry([e[1].elapsed_time(e[2]) for e in ev], 2 * k + 26, n),
                    "gs_grad_sqnorm": _kernel_entry([e[0].elapsed_time(e[1]) for e in ev], 2 * k, n),
                    "note": "one tensor set reused every iteration (warm caches); not the reported figures"}

    step_bytes = n * (2 * k + 26)
    cache_protocol = (f"cold: rotation over {nsets} independent tensor sets of {working_set / 1e6:.0f} MB each, one per "
                      f"iteration ({nsets * working_set / 1e9:.2f} GB in all against a {CACHE_BYTES >> 20} MB last-level cache)"
                      if nsets > 1 else
                      f"one tensor set: its {working_set / 1e9:.1f} GB working set is {working_set / CACHE_BYTES:.0f}x the "
                      f"{CACHE_BYTES >> 20} MB last-level cache, so every pass is cold")
    out = _base_record(wl, props, n * args.steps / elapsed, args.steps, args.warmup, elapsed / args.steps * 1e3,
                       {"input_gen_s": round(t_gen, 2), "tensor_sets": nsets, "cache_protocol": cache_protocol})
    out["timing"] = {"per_step": _stats(both_l), "protocol": "HIP events around every launch on the launch stream; "
                     "mean, median and minimum over the timed steps; `value` is wall clock over all of them"}
    traffic = MEASURED_TRAFFIC_BYTES.get(wl.name)
    out["roofline"] = {"bound": "hbm", "kernel": "gs_accum_adamw", "achieved": k_step["GBps"], "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": k_step["frac"], "traffic": traffic,
                       "traffic_source": (None if traffic is None else
                                          "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel on this workload, from the "
                                          "summary under profiles/ (a stored figure, not measured by this run)"),
                       "algorithmic_bytes_per_launch": step_bytes, "avg_launch_ms": k_step["avg_ms"],
                       "median_launch_ms": k_step["median_ms"], "min_launch_ms": k_step["min_ms"],
                       "frac_median": k_step["GBps_median"] / HBM_PEAK_GBS, "frac_best": k_step["GBps_best"] / HBM_PEAK_GBS,
                       "params_per_s": n / (k_step["avg_ms"] * 1e-3)}
    out["kernels"] = {"gs_accum_adamw": k_step, "gs_grad_sqnorm": k_norm}
    if warm_ref:
        out["warm_cache_reference"] = warm_ref
    if not full:
        out["cpu_baseline"] = None
        return out

    # the staged two-pass variant of the same step (norm pass leaves the fp32 sum behind): reported
    # beside the headline, never as `value`
    acc = torch.empty(n, dtype=torch.float32, device=dev)
    ws_big = torch.empty(gs.gs_sqnorm_workspace_bytes_for(n), dtype=torch.uint8, device=dev)   # fastest shape
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(max(1, args.warmup)):
        gs.gs_grad_accum_sqnorm(grads, 0, n, acc, sq, ws_big)
        gs.gs_adamw_from_acc(p, m, v, w, acc, 0, n, hp_at(i), sq)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        ev2[i][0].record()
        gs.gs_grad_accum_sqnorm(grads, 0, n, acc, sq, ws_big)
        ev2[i][1].record()
        gs.gs_adamw_from_acc(p, m, v, w, acc, 0, n, hp_at(i), sq)
        ev2[i][2].record()
    torch.cuda.synchronize()
    staged_elapsed = time.perf_counter() - t1

    # accumulate as you go: one micro-batch added into the resident fp32 buffer per call, the
    # last call also reducing the norm; then the step from the buffer
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        out_ms = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            out_ms.append(e0.elapsed_time(e1))
        return out_ms
    add_first = timed(lambda: gs.gs_accum_add(acc, grads[0], True, 0, n), args.steps)
    add = timed(lambda: gs.gs_accum_add(acc, grads[1 % k], False, 0, n), args.steps)
    add_norm = timed(lambda: gs.gs_accum_add(acc, grads[k - 1], False, 0, n, sq, ws_big), args.steps)
    acc_norm = timed(lambda: gs.gs_acc_sqnorm(acc, 0, n, sq, ws), args.steps)
    noalloc_norm = timed(lambda: gs.gs_grad_sqnorm_noalloc(grads, 0, n, sq), args.steps)
    del acc

    # speculative single pass (c = 1 step + norm in one read of the gradients), out of place with
    # ping-pong state buffers; on these workloads the norm always exceeds max_norm, so a caller would
    # have to redo the step -- the figure shows what the pass costs when the guess holds
    A_ = [p, m, v]
    B_ = [torch.empty_like(p), torch.empty_like(m), torch.empty_like(v)]
    for i in range(max(1, args.warmup)):
        gs.gs_accum_adamw_spec(*A_, *B_, w, grads, 0, n, hp_at(i), sq, ws_big)
        A_, B_ = B_, A_
    torch.cuda.synchronize()
    es = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    es[0].record()
    for i in range(args.steps):
        gs.gs_accum_adamw_spec(*A_, *B_, w, grads, 0, n, hp_at(i), sq, ws_big)
        A_, B_ = B_, A_
        es[i + 1].record()
    torch.cuda.synchronize()
    spec_l = [es[i].elapsed_time(es[i + 1]) for i in range(args.steps)]
    if A_[0] is not p:                       # leave the states in the caller-visible p, m, v
        for dst, src in zip((p, m, v), A_):
            dst.copy_(src)
    del B_, A_

    # what this device gives simpler traffic, and the step's own mix of streams without arithmetic
    cp_dst = torch.empty_like(p)
    copy_ms = _stats(timed(lambda: cp_dst.copy_(p), max(4, args.steps // 2)))["avg_ms"]
    del cp_dst
    copy_gbs = 8 * n / (copy_ms * 1e-3) / 1e9
    read_gbs = n * 4 / (_stats(acc_norm)["avg_ms"] * 1e-3) / 1e9
    achieved = k_step["GBps"]
    achievable = {"device_copy_GBps": copy_gbs, "frac_of_device_copy": achieved / copy_gbs,
                  "read_only_GBps": read_gbs, "frac_of_read_only": achieved / read_gbs,
                  "note": "measured here after the timed region: torch's device-to-device copy of one fp32 state array "
                          "(bytes read + written), a read-only pass (gs_acc_sqnorm)"}
    if not args.no_ceiling:
        block = 128 if k >= 15 else 64           # the step kernel's own workgroup size for this k
        try:
            mix = same_mix_ceiling(torch, grads, p, m, v, w, n, k, max(4, args.steps // 2), block)
        except Exception as exc:                 # the probe library is an extra: its absence must not cost the line
            mix = None
            achievable["same_mix_error"] = f"{type(exc).__name__}: {exc}"
    if not args.no_ceiling and mix is not None:
        achievable.update(mix)
        achievable["frac_of_same_mix"] = achieved / mix["same_mix_ceiling_GBps"]
        achievable["frac_of_read_kernel_beside_write_kernel"] = achieved / mix["same_mix_read_kernel_beside_write_kernel_GBps"]
        achievable["note"] += ("; and kernels with the step's own mix of streams and no arithmetic (probe/gs_mixprobe.hip): "
                               "in the step kernel's shape and with all loads in flight (same_mix_ceiling = the better of "
                               "the two single kernels), and split into a read-only kernel running beside a write-only "
                               "kernel on a second stream (the same bytes issued from separate workgroups)")
    out["roofline"]["achievable"] = achievable
    out["staged_two_pass"] = {
        "params_per_s": n * args.steps / staged_elapsed, "ms_per_step": staged_elapsed / args.steps * 1e3,
        "gs_grad_accum_sqnorm": _kernel_entry([e[0].elapsed_time(e[1]) for e in ev2], 2 * k + 4, n),
        "gs_adamw_from_acc": _kernel_entry([e[1].elapsed_time(e[2]) for e in ev2], 30, n),
        "note": "same results bit for bit; (2k+4)+30 B/param in total instead of 2k+(2k+26)"}
    out["accumulate_as_you_go"] = {
        "gs_accum_add_first": _kernel_entry(add_first, 6, n), "gs_accum_add": _kernel_entry(add, 10, n),
        "gs_accum_add_with_norm": _kernel_entry(add_norm, 10, n), "gs_acc_sqnorm": _kernel_entry(acc_norm, 4, n),
        "note": "one call per micro-batch into the resident fp32 buffer; the step then runs gs_adamw_from_acc"}
    out["no_alloc_norm"] = dict(_kernel_entry(noalloc_norm, 2 * k, n),
                                note="gs_grad_sqnorm_noalloc: partials in the library's fixed device array")
    sp = _kernel_entry(spec_l, 2 * k + 26, n)
    sp.update({"params_per_s": n / (sp["avg_ms"] * 1e-3),
               "note": "gs_accum_adamw_spec, out of place, step with c=1 plus squared norm; valid as the whole step only "
                       "when no clipping turns out to be needed"})
    out["speculative_single_pass"] = sp
    out["cpu_baseline"] = cpu
    return out


def bench_k_sweep(args, wl):
    """The two kernels on one resident layer of the workload's shape as the number of bf16 gradient
    buffers goes from 1 to 32: how the achieved bandwidth moves with the share of gradient reads
    (2k of 2k+26 bytes) and with the kernel shapes chosen per k."""
    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    dev = "cuda:0"
    props = torch.cuda.get_device_properties(0)
    n = I.layer_numel(wl.h)
    ks = (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 15, 16, 20, 24, 32)
    p, m, v = I.make_states(n, wl.seed, dev)
    grads = I.make_grads(n, max(ks), wl.grad_sigma, wl.seed, dev)
    w = torch.zeros(n, dtype=torch.bfloat16, device=dev)
    sq = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
    rows = {}
    for k in ks:
        g = grads[:k]
        hp = gs.HParams(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.max_grad_norm, wl.step)
        for _ in range(max(2, args.warmup)):
            gs.gs_grad_sqnorm(g, 0, n, sq, ws)
            gs.gs_accum_adamw(p, m, v, w, g, 0, n, hp, sq)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        for i in range(args.steps):
            ev[i][0].record()
            gs.gs_grad_sqnorm(g, 0, n, sq, ws)
            ev[i][1].record()
            gs.gs_accum_adamw(p, m, v, w, g, 0, n, hp, sq)
            ev[i][2].record()
        torch.cuda.synchronize()
        rows[str(k)] = {"gs_accum_adamw": _kernel_entry([e[1].elapsed_time(e[2]) for e in ev], 2 * k + 26, n),
                        "gs_grad_sqnorm": _kernel_entry([e[0].elapsed_time(e[1]) for e in ev], 2 * k, n),
                        "read_share_of_step_bytes": (2 * k + 12) / (2 * k + 26)}
    best = max(rows, key=lambda kk: rows[kk]["gs_accum_adamw"]["frac"])
    rec = _base_record(wl, props, n / (rows[str(wl.k)]["gs_accum_adamw"]["avg_ms"] * 1e-3) if str(wl.k) in rows else 0.0,
                       args.steps, args.warmup, rows[str(wl.k)]["gs_accum_adamw"]["avg_ms"] if str(wl.k) in rows else 0.0,
                       {"n_params": n, "layers": 1, "sweep": "k_grad_buffers 1..32"})
    rec["metric"] = "params/s, gs_accum_adamw alone at the workload's k (k sweep)"
    rec["k_sweep"] = rows
    rec["best_k_for_step_frac"] = int(best)
    rec["roofline"] = None
    rec["cpu_baseline"] = None
    return rec


def _brief(rec, keys):
    return {k: rec[k] for k in keys if k in rec}


def streamed_short(args):
    """Short form of the host-resident workload (fewer layers and passes, same chunking and
    pipeline).  Run FIRST in the process: the staged pipeline's rate depends on which hardware
    queues the runtime gives the context's three streams, and streams created earlier in the
    process change that assignment (upload and download on one queue halve the rate)."""
    import gc

    import torch

    from paper_2512_17570_amd import inputs as I

    res = {}
    t0 = time.perf_counter()
    r = bench_streamed(args, I.WORKLOADS["gpt65b_8layers_streamed_k8"], brief=True)
    res["gpt65b_8layers_streamed_k8"] = {
        "layers": r["config"]["layers"], "layers_in_workload": r["config"]["layers_in_workload"],
        "n_params": r["config"]["n_params"], "passes_timed": r["steps"],
        "staged": {"params_per_s": r["value"], "ms_per_pass": r["ms_per_step"],
                   "copies_overlap_check": r["config"]["copies_overlap_check"],
                   "GBps_per_direction": r["roofline"]["achieved"], "frac_of_link": r["roofline"]["frac"]},
        "in_place": _brief(r["in_place"], ("params_per_s", "ms_per_step", "GBps_per_direction", "frac_of_link", "stream_cus")),
        "link": _brief(r["roofline"], ("h2d_only_GBps", "d2h_only_GBps", "duplex_copy_probe_GBps_per_direction",
                                       "params_per_s_bound")),
        "note": "short form of --workload gpt65b_8layers_streamed_k8: fewer layers and passes, same chunking and pipeline; "
                "run first in the process, before any other stream exists (the staged pipeline's rate depends on which "
                "hardware queues its three streams are given)",
        "wall_s": round(time.perf_counter() - t0, 1)}
    del r
    gc.collect()
    torch.cuda.empty_cache()
    return res["gpt65b_8layers_streamed_k8"]


def other_workloads(args):
    """The other configurations of the workload list, each in a short run, for the record that the
    default invocation prints: the two smaller layers and the GPT-30B-shaped one (norm + step) and the
    split step of the GPT-175B-shaped layer beside a GEMM (the host-resident one is streamed_short)."""
    import gc

    import torch

    from paper_2512_17570_amd import inputs as I

    res = {}

    def free():
        gc.collect()
        torch.cuda.empty_cache()

    for name in ("gpt_h1024_k4", "gpt_h4096_k8", "gpt30b_layer_h7168_k16"):
        t0 = time.perf_counter()
        try:
            r = bench_resident(args, I.WORKLOADS[name], full=False)
        except Exception as exc:                       # recorded, not fatal (see main)
            res[name] = {"error": f"{type(exc).__name__}: {exc}"}
            free()
            continue
        res[name] = {"params_per_s": r["value"], "ms_per_step": r["ms_per_step"], "n_params": r["config"]["n_params"],
                     "k": r["config"]["k_grad_buffers"], "cache_protocol": r["config"]["cache_protocol"],
                     "per_step": r["timing"]["per_step"], "kernels": r["kernels"], "wall_s": None}
        if "warm_cache_reference" in r:
            res[name]["warm_cache_reference"] = r["warm_cache_reference"]
        res[name]["wall_s"] = round(time.perf_counter() - t0, 1)
        del r
        free()
    t0 = time.perf_counter()
    try:
        r = bench_split(args, I.WORKLOADS["gpt175b_layer_h12288_k8_split"], brief=True)
    except Exception as exc:
        res["gpt175b_layer_h12288_k8_split"] = {"error": f"{type(exc).__name__}: {exc}"}
        free()
        return res
    sp = r["split"]
    res["gpt175b_layer_h12288_k8_split"] = {
        "n_params": r["config"]["n_params"], "k": r["config"]["k_grad_buffers"], "split_point": r["config"]["split_point"],
        "full_ms": sp["full_ms"], "immediate_ms": sp["immediate_ms"], "deferred_alone_ms": sp["deferred_alone_ms"],
        "full_GBps": r["roofline"]["achieved"], "full_frac": r["roofline"]["frac"],
        "split_vs_full": (sp["immediate_ms"] + sp["deferred_alone_ms"]) / sp["full_ms"],
        "split_equals_full_bitwise": sp["split_equals_full_bitwise"],
        "gemm": r["config"]["gemm"], "gemms_per_deferred_step": r["config"]["gemms_per_deferred_step"],
        "gemm_alone_ms": sp["gemm_alone_ms"], "gemm_alone_TFLOPs": sp["gemm_alone_TFLOPs"],
        "deferred_beside_gemm_ms": sp["deferred_concurrent_ms"], "gemm_beside_deferred_ms": sp["gemm_concurrent_ms"],
        "deferred_slowdown": sp["deferred_slowdown"], "gemm_slowdown": sp["gemm_slowdown"],
        "concurrent_wall_ms_per_iter": sp["concurrent_wall_ms_per_iter"], "serial_ms_per_iter": sp["serial_ms_per_iter"],
        "wall_s": round(time.perf_counter() - t0, 1)}
    del r
    free()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (no sharding or collectives); --gpus {args.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2512_17570_amd import gs  # noqa: F401  (fails loudly if libgs.so is missing)
    from paper_2512_17570_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.workload not in I.WORKLOADS:
        print(f"unknown workload {args.workload}; have {list(I.WORKLOADS)}", file=sys.stderr)
        sys.exit(2)
    wl = I.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    if args.k_sweep:
        print(json.dumps(bench_k_sweep(args, wl)))
        return
    if "immediate_frac" in wl.extra:
        rec = bench_split(args, wl)
    elif "host_share" in wl.extra:
        rec = bench_tiered(args, wl)
    elif "chunk_elems" in wl.extra:
        rec = bench_streamed(args, wl)
    else:
        # the short runs of the other workloads are extras: a failure in one of them (a host that cannot
        # pin enough memory, say) is recorded in its place and never costs the headline line
        def guarded(fn):
            try:
                return fn(args)
            except (Exception, SystemExit) as exc:
                torch.cuda.synchronize()
                return {"error": f"{type(exc).__name__}: {exc}"}

        others = wl.name == HEADLINE and not args.no_other_workloads
        streamed = guarded(streamed_short) if others else None
        rec = bench_resident(args, wl, full=True)
        if others:
            import gc
            gc.collect()
            torch.cuda.empty_cache()
            t0 = time.perf_counter()
            rec["other_workloads"] = guarded(other_workloads)
            rec["other_workloads"]["gpt65b_8layers_streamed_k8"] = streamed
            rec["other_workloads"]["wall_s"] = round(time.perf_counter() - t0 + streamed.get("wall_s", 0.0), 1)
    if NOTES:
        rec["notes"] = sorted(set(NOTES))
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
