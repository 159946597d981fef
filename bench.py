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
MEASURED_TRAFFIC_BYTES = {"gpt65b_layer_h8192_k16": 46_714_044_211}   # profiles/gs_step_gpt65b_layer_h8192_k16.txt


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
                     "params_per_s": n / (step_ms * 1e-3)},
        "kernels": {
            "gs_accum_adamw": {"avg_ms": step_ms, "bytes_per_param": 2 * k + 26, "GBps": achieved},
            "gs_grad_sqnorm": {"avg_ms": norm_ms, "bytes_per_param": 2 * k,
                               "GBps": norm_bytes / (norm_ms * 1e-3) / 1e9,
                               "frac": norm_bytes / (norm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        },
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
