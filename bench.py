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
measured with HIP events on the launch stream, against the 8 TB/s HBM peak.  `cpu_baseline`
times the CPU oracle on a bounded sample of the same tensors on the host's cores.
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
MEASURED_TRAFFIC_BYTES = {"gpt65b_layer_h8192_k16": 46_712_699_261,    # profiles/gs_step_gpt65b_layer_h8192_k16.txt
                          "gpt_h4096_k8": 8_458_116_813}               # profiles/gs_step_gpt_h4096_k8.txt


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    """Time the oracle (norm pass + fused step, as it stands) on the first `sample` elements,
    split over the host's cores in disjoint ranges."""
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
    bounds = [sample * i // cores for i in range(cores + 1)]
    O.lib()

    def norm_part(i):
        return O.grad_sqnorm(h_g, bounds[i], bounds[i + 1])

    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        S = sum(ex.map(norm_part, range(cores)))
        c = O.clip_coef(S, hp.max_grad_norm)
        list(ex.map(lambda i: O.accum_adamw(h_p, h_m, h_v, h_w, h_g, ohp, c, bounds[i], bounds[i + 1]), range(cores)))
    dt = time.perf_counter() - t0
    return {"value": sample / dt, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample} of {wl.n} parameters of the same tensors, norm pass + fused step, "
                      f"{cores} threads over disjoint ranges, {dt:.2f} s wall"}


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


def bench_split(args, wl):
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
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
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
    for ncu in (cus // 2, (3 * cus) // 4):
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

    def sequence(step_stream, overlap, reps):
        def once():
            evs = []
            with torch.cuda.stream(step_stream):
                for _ in range(seq_layers):
                    deferred(step_stream)
                    ev = torch.cuda.Event()
                    ev.record(step_stream)
                    evs.append(ev)
            with torch.cuda.stream(sa):
                if not overlap:
                    sa.wait_event(evs[-1])
                for i in range(seq_layers):
                    if overlap:
                        sa.wait_event(evs[i])
                    forward_layer()
            # the next iteration's steps follow this iteration's forward
            done = torch.cuda.Event()
            done.record(sa)
            step_stream.wait_event(done)
        once()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            once()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

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
           "serial_ms": sequence(sb, False, seq_reps),
           "overlapped_all_cus_ms": sequence(sb, True, seq_reps)}
    for ncu in (cus // 4, cus // 2):
        raw = gs.gs_cu_stream_create(ncu)
        sc = torch.cuda.ExternalStream(raw)
        seq[f"overlapped_{ncu}_cus_ms"] = sequence(sc, True, seq_reps)
        del sc
        gs.gs_cu_stream_destroy(raw)
    seq["bound_ms"] = t_def + seq_layers * t_fwd_layer      # first step exposed, everything else hidden
    seq["note"] = ("forward of layer i waits for layer i's deferred step; steps run in layer order on their own stream. "
                   "bound = one exposed deferred step + the forwards at their solo speed")

    bpp = 2 * k + 26
    rec = _base_record(wl, props, n / ((t_imm + t_def) * 1e-3), args.steps, args.warmup, t_imm + t_def,
                       {"split_point": s_pt, "immediate_frac": wl.extra["immediate_frac"],
                        "gemm": f"bf16 {tokens}x{wl.h} @ {wl.h}x{wl.h}", "gemms_per_deferred_step": reps_gemm})
    rec["roofline"] = {"bound": "hbm", "kernel": "gs_accum_adamw (full range)", "achieved": n * bpp / (t_full * 1e-3) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": n * bpp / (t_full * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "traffic": None, "algorithmic_bytes_per_launch": n * bpp, "avg_launch_ms": t_full}
    gemm_flop = 2.0 * tokens * wl.h * wl.h
    rec["split"] = {
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
    print(json.dumps(rec))


def bench_streamed(args, wl):
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
        for i in range(args.warmup):
            one_pass(i)
        t0 = time.perf_counter()
        for i in range(args.steps):
            one_pass(args.warmup + i)
        return (time.perf_counter() - t0) / args.steps

    # the configuration as named: 2^26-element chunks, upload | kernel in an HBM slot | download
    ctx = gs.gs_stream_ctx_create(chunk, args.slots)
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
    up, dn = torch.cuda.Stream(), torch.cuda.Stream()
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
    h2d_only_gbs = copy_pass(32, True, False)
    d2h_only_gbs = copy_pass(32, False, True)
    duplex_dir_gbs = copy_pass(48, True, True)
    del stage

    rec = _base_record(wl, props, n / per, args.steps, args.warmup, per * 1e3,
                       {"layers_pinned": layers, "n_params": n, "chunk_elems": chunk, "slots": args.slots,
                        "host_pinned_bytes": 12 * n, "device_staging_bytes": args.slots * 3 * (chunk + 64) * 4})
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
    print(json.dumps(rec))
    for t, ptr in bufs:
        gs.gs_pinned_free(ptr)


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
        print(json.dumps(rec))
    finally:
        for lf in fds:
            for fd in lf:
                os.close(fd)
        shutil.rmtree(root, ignore_errors=True)
        for bufs in hosts:
            for _, ptr in bufs:
                gs.gs_pinned_free(ptr)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (no sharding or collectives); --gpus {args.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2512_17570_amd import gs
    from paper_2512_17570_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.workload not in I.WORKLOADS:
        print(f"unknown workload {args.workload}; have {list(I.WORKLOADS)}", file=sys.stderr)
        sys.exit(2)
    wl = I.WORKLOADS[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if "immediate_frac" in wl.extra:
        return bench_split(args, wl)
    if "host_share" in wl.extra:
        return bench_tiered(args, wl)
    if "chunk_elems" in wl.extra:
        return bench_streamed(args, wl)
    props = torch.cuda.get_device_properties(0)

    t_gen = time.perf_counter()
    p, m, v, grads = I.make_workload_tensors(wl, dev)
    w = torch.zeros(wl.n, dtype=torch.bfloat16, device=dev)
    sq = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    n, k = wl.n, wl.k

    def hp_at(i):
        return gs.HParams(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.max_grad_norm, wl.step + i)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, p, m, v, grads, hp_at(0), args.cpu_sample)

    def one_step(i, evs=None):
        if evs:
            evs[0].record()
        gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
        if evs:
            evs[1].record()
        gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp_at(i), sq)
        if evs:
            evs[2].record()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    norm_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    step_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps

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
    st_norm_ms = sum(e[0].elapsed_time(e[1]) for e in ev2) / args.steps
    st_step_ms = sum(e[1].elapsed_time(e[2]) for e in ev2) / args.steps

    # accumulate as you go: one micro-batch added into the resident fp32 buffer per call, the
    # last call also reducing the norm; then the step from the buffer
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    add_first_ms = timed(lambda: gs.gs_accum_add(acc, grads[0], True, 0, n), args.steps)
    add_ms = timed(lambda: gs.gs_accum_add(acc, grads[1 % k], False, 0, n), args.steps)
    add_norm_ms = timed(lambda: gs.gs_accum_add(acc, grads[k - 1], False, 0, n, sq, ws_big), args.steps)
    acc_norm_ms = timed(lambda: gs.gs_acc_sqnorm(acc, 0, n, sq, ws), args.steps)
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
    spec_ms = es[0].elapsed_time(es[-1]) / args.steps
    del B_, A_
    # what this device gives a plain device-to-device copy of one state array (read + written bytes):
    # the practical ceiling for a kernel that, like the step, both reads and writes
    cp_dst = torch.empty_like(p)
    copy_ms = timed(lambda: cp_dst.copy_(p), max(4, args.steps))
    del cp_dst
    copy_gbs = 8 * n / (copy_ms * 1e-3) / 1e9
    step_bytes = n * (2 * k + 26)
    norm_bytes = n * 2 * k
    achieved = step_bytes / (step_ms * 1e-3) / 1e9
    out = {
        "metric": "params/s, fused grad-norm + accumulate + AdamW step",
        "value": n * args.steps / elapsed,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "h": wl.h, "layers": wl.layers, "n_params": n, "k_grad_buffers": k,
                   "grad_dtype": "bf16", "state_dtype": "f32", "clip_max_norm": wl.max_grad_norm,
                   "device": props.name, "compute_units": props.multi_processor_count,
                   "hbm_bytes": props.total_memory, "input_gen_s": round(t_gen, 2)},
        "roofline": {"bound": "hbm", "kernel": "gs_accum_adamw", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name),
                     "algorithmic_bytes_per_launch": step_bytes, "avg_launch_ms": step_ms,
                     "params_per_s": n / (step_ms * 1e-3),
                     "achievable": {"device_copy_GBps": copy_gbs, "frac_of_device_copy": achieved / copy_gbs,
                                    "read_only_GBps": n * 4 / (acc_norm_ms * 1e-3) / 1e9,
                                    "frac_of_read_only": achieved / (n * 4 / (acc_norm_ms * 1e-3) / 1e9),
                                    "note": "measured here after the timed region: a device-to-device copy of one fp32 "
                                            "state array (bytes read + written) and a read-only pass (gs_acc_sqnorm)"}},
        "kernels": {
            "gs_accum_adamw": {"avg_ms": step_ms, "bytes_per_param": 2 * k + 26, "GBps": achieved},
            "gs_grad_sqnorm": {"avg_ms": norm_ms, "bytes_per_param": 2 * k,
                               "GBps": norm_bytes / (norm_ms * 1e-3) / 1e9,
                               "frac": norm_bytes / (norm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        },
        "staged_two_pass": {
            "params_per_s": n * args.steps / staged_elapsed, "ms_per_step": staged_elapsed / args.steps * 1e3,
            "gs_grad_accum_sqnorm": {"avg_ms": st_norm_ms, "bytes_per_param": 2 * k + 4,
                                     "GBps": n * (2 * k + 4) / (st_norm_ms * 1e-3) / 1e9},
            "gs_adamw_from_acc": {"avg_ms": st_step_ms, "bytes_per_param": 30,
                                  "GBps": n * 30 / (st_step_ms * 1e-3) / 1e9},
            "note": "same results bit for bit; (2k+4)+30 B/param in total instead of 2k+(2k+26)"},
        "accumulate_as_you_go": {
            "gs_accum_add_first": {"avg_ms": add_first_ms, "bytes_per_param": 6,
                                   "GBps": n * 6 / (add_first_ms * 1e-3) / 1e9},
            "gs_accum_add": {"avg_ms": add_ms, "bytes_per_param": 10, "GBps": n * 10 / (add_ms * 1e-3) / 1e9},
            "gs_accum_add_with_norm": {"avg_ms": add_norm_ms, "bytes_per_param": 10,
                                       "GBps": n * 10 / (add_norm_ms * 1e-3) / 1e9},
            "gs_acc_sqnorm": {"avg_ms": acc_norm_ms, "bytes_per_param": 4, "GBps": n * 4 / (acc_norm_ms * 1e-3) / 1e9},
            "note": "one call per micro-batch into the resident fp32 buffer; the step then runs gs_adamw_from_acc"},
        "speculative_single_pass": {"avg_ms": spec_ms, "bytes_per_param": 2 * k + 26,
                                    "GBps": step_bytes / (spec_ms * 1e-3) / 1e9, "params_per_s": n / (spec_ms * 1e-3),
                                    "note": "gs_accum_adamw_spec, out of place, step with c=1 plus squared norm; "
                                            "valid as the whole step only when no clipping turns out to be needed"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
