"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module serves both the HIP path and the CPU oracle and therefore holds none of the
method's arithmetic: it only draws random tensors (torch's seeded generators, on whichever
device is asked for) and lays them out as one flat GPT layer.

Shapes follow the paper's model table (Table 2: GPT-30B/65B/175B with hidden sizes
7168 / 8192 / 12288) and its count of about 8.05e8 parameters for one GPT-65B layer
(Sec. 3.4).  A layer is flattened as
    ln1.w ln1.b | qkv.w[h,3h] qkv.b | out.w[h,h] out.b | ln2.w ln2.b |
    fc1.w[h,4h] fc1.b | fc2.w[4h,h] fc2.b
which gives 12 h^2 + 13 h elements.  The step is element-wise, so the order only fixes the
seed -> value mapping.

Value distributions (the paper trains on the Pile, which is not available; these synthetic
tensors stand in for real weights and gradients, whose values do not change the cost of the
step): master weights ~ N(0, 0.02), momentum ~ N(0, 1e-3), variance = N(0, 1e-3)^2,
k bf16 micro-batch gradients ~ N(0, sigma), optionally with a sparse set of outliers scaled
up so that clipping fires.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch


def layer_numel(h: int, ffn: int | None = None) -> int:
    """Flat parameter count of one GPT layer with hidden size h (ffn defaults to 4h)."""
    ffn = 4 * h if ffn is None else ffn
    return (2 * h) + (h * 3 * h + 3 * h) + (h * h + h) + (2 * h) + (h * ffn + ffn) + (ffn * h + h)


def layer_segments(h: int, ffn: int | None = None):
    """(name, numel) of each tensor of the flat layer, in flat order."""
    ffn = 4 * h if ffn is None else ffn
    return [("ln1.w", h), ("ln1.b", h), ("qkv.w", h * 3 * h), ("qkv.b", 3 * h),
            ("out.w", h * h), ("out.b", h), ("ln2.w", h), ("ln2.b", h),
            ("fc1.w", h * ffn), ("fc1.b", ffn), ("fc2.w", ffn * h), ("fc2.b", h)]


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: a stack of `layers` GPT layers of hidden size h."""
    name: str
    h: int
    k: int
    grad_sigma: float
    step: int
    layers: int = 1
    outlier_frac: float = 0.0      # fraction of gradient entries scaled by outlier_scale
    outlier_scale: float = 100.0
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    max_grad_norm: float = 1.0
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.layers * layer_numel(self.h)


WORKLOADS = {
    # small case the oracle finishes in seconds
    "gpt_h1024_k4": Workload("gpt_h1024_k4", h=1024, k=4, grad_sigma=1e-3, step=10),
    # clipping fires: 0.1 % of entries scaled x100
    "gpt_h4096_k8": Workload("gpt_h4096_k8", h=4096, k=8, grad_sigma=1e-3, step=100, outlier_frac=1e-3),
    # headline bandwidth workload: one GPT-65B-shaped layer
    "gpt65b_layer_h8192_k16": Workload("gpt65b_layer_h8192_k16", h=8192, k=16, grad_sigma=5e-4, step=100),
    # one GPT-30B-shaped layer (Table 2: hidden 7168), second resident workload
    "gpt30b_layer_h7168_k16": Workload("gpt30b_layer_h7168_k16", h=7168, k=16, grad_sigma=5e-4, step=100),
    # GPT-175B-shaped layer, split step (40 % immediate / 60 % deferred)
    "gpt175b_layer_h12288_k8_split": Workload("gpt175b_layer_h12288_k8_split", h=12288, k=8, grad_sigma=5e-4,
                                              step=100, extra={"immediate_frac": 0.4, "gemm_tokens": 4096}),
    # eight GPT-65B layers with host-resident states, streamed in 2^26-element chunks
    "gpt65b_8layers_streamed_k8": Workload("gpt65b_8layers_streamed_k8", h=8192, k=8, grad_sigma=1e-3, step=100,
                                           layers=8, extra={"chunk_elems": 1 << 26}),
    # two GPT-65B layers, half of each layer's states in pinned host memory and half in files
    "gpt65b_2layers_tiered_k8": Workload("gpt65b_2layers_tiered_k8", h=8192, k=8, grad_sigma=1e-3, step=100,
                                         layers=2, extra={"chunk_elems": 1 << 24, "host_share": 0.5}),
}

_CHUNK = 1 << 24


def _gen(seed: int, stream_id: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(stream_id) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def normal_f32(n: int, sigma: float, seed: int, stream_id: int, device="cpu", square: bool = False,
               out: torch.Tensor | None = None) -> torch.Tensor:
    """n values of N(0, sigma) (or their squares), fp32, drawn chunk-wise from one seeded stream."""
    g = _gen(seed, stream_id, device)
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        x = torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32) * sigma
        if square:
            x = x * x
        out[lo:hi].copy_(x)
    return out


def make_states(n: int, seed: int = 0, device="cpu"):
    """(p, m, v) fp32: p ~ N(0,0.02), m ~ N(0,1e-3), v = N(0,1e-3)^2."""
    p = normal_f32(n, 0.02, seed, 1, device)
    m = normal_f32(n, 1e-3, seed, 2, device)
    v = normal_f32(n, 1e-3, seed, 3, device, square=True)
    return p, m, v


def make_grads(n: int, k: int, sigma: float, seed: int = 0, device="cpu",
               outlier_frac: float = 0.0, outlier_scale: float = 100.0):
    """k bf16 micro-batch gradient buffers ~ N(0, sigma); a fraction `outlier_frac` of the
    entries is multiplied by `outlier_scale` before the cast to bf16."""
    grads = []
    for j in range(k):
        g = _gen(seed, 100 + j, device)
        out = torch.empty(n, dtype=torch.bfloat16, device=device)
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            x = torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32) * sigma
            if outlier_frac > 0.0:
                u = torch.rand(hi - lo, generator=g, device=device, dtype=torch.float32)
                x = torch.where(u < outlier_frac, x * outlier_scale, x)
            out[lo:hi].copy_(x.to(torch.bfloat16))
        grads.append(out)
    return grads


def make_workload_tensors(wl: Workload, device="cpu", n: int | None = None):
    """All tensors of a workload (optionally truncated to the first n elements)."""
    n = wl.n if n is None else n
    p, m, v = make_states(n, wl.seed, device)
    grads = make_grads(n, wl.k, wl.grad_sigma, wl.seed, device, wl.outlier_frac, wl.outlier_scale)
    return p, m, v, grads


def bf16_bits(t: torch.Tensor):
    """numpy uint16 view of a CPU bf16 tensor's bit patterns."""
    import numpy as np
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
