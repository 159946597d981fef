"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding, run the
CPU oracle on the same bytes, compare to the stated tolerances.

Tolerances (GPU vs oracle, same seeded inputs):
  fp32 p/m/v : within 4 fp32 ulp OR 1e-6 relative
  bf16 w     : within 1 bf16 ulp of the oracle's w, and exactly bf16_rne of the GPU's own p'
  sqnorm     : within 1e-5 relative
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import gs_oracle as O
from paper_2512_17570_amd import gs
from paper_2512_17570_amd import inputs as I
from tolerances import f64_truth_check  # noqa: F401  (re-exported for the GPU tests)

DEV = "cuda:0"


def np_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().copy()


def np_bf16(t: torch.Tensor) -> np.ndarray:
    return I.bf16_bits(t).copy()


def ohp(hp: gs.HParams) -> O.HParams:
    return O.HParams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.max_grad_norm, hp.step)


def ulp_key(x: np.ndarray) -> np.ndarray:
    i = x.view(np.int32).astype(np.int64)
    return np.where(i < 0, -(i & 0x7FFFFFFF), i)


def assert_f32_close(got: np.ndarray, want: np.ndarray, name: str):
    """4 fp32 ulp or 1e-6 relative; NaNs must coincide."""
    gn, wn = np.isnan(got), np.isnan(want)
    assert np.array_equal(gn, wn), f"{name}: NaN pattern differs"
    ok = ~gn
    g, w = got[ok], want[ok]
    ul = np.abs(ulp_key(g) - ulp_key(w))
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.abs(g.astype(np.float64) - w.astype(np.float64)) / np.abs(w.astype(np.float64))
    rel = np.where(g == w, 0.0, rel)
    bad = ~((ul <= 4) | (rel <= 1e-6))
    assert not bad.any(), f"{name}: {bad.sum()} elements out of tolerance, max ulp {ul.max()}, max rel {np.nanmax(rel)}"
    return int(ul.max()) if ul.size else 0


def assert_bf16_close(got: np.ndarray, want: np.ndarray, name: str):
    """Within 1 bf16 ulp (distance of the monotone integer keys of the 16-bit patterns)."""
    def key(b):
        i = b.astype(np.int32)
        return np.where(i & 0x8000, -(i & 0x7FFF), i)
    def isnan(b):
        return ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)
    gn, wn = isnan(got), isnan(want)
    assert np.array_equal(gn, wn), f"{name}: NaN pattern differs"
    d = np.abs(key(got) - key(want))[~gn]
    assert d.size == 0 or d.max() <= 1, f"{name}: max bf16 ulp distance {d.max()}"
    return int(d.max()) if d.size else 0


def assert_w_is_rne_of_p(p_dev: torch.Tensor, w_dev: torch.Tensor, lo: int, hi: int):
    """a6: the emitted working weight is exactly bf16_rne of the GPU's own new master weight
    (torch's cast is the independent rounding)."""
    want = p_dev[lo:hi].to(torch.bfloat16)
    got = w_dev[lo:hi]
    nan = torch.isnan(want)
    assert torch.equal(torch.isnan(got), nan)
    assert torch.equal(got[~nan].view(torch.int16), want[~nan].view(torch.int16))


class DeviceCase:
    """One set of device tensors + the matching host copies of the INPUTS."""

    def __init__(self, n: int, k: int, seed: int = 0, sigma: float = 1e-3, outlier_frac: float = 0.0,
                 keep_host: bool = True):
        self.n, self.k = n, k
        self.p, self.m, self.v = I.make_states(n, seed, DEV)
        self.grads = I.make_grads(n, k, sigma, seed, DEV, outlier_frac)
        self.w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
        self.sq = torch.zeros(1, dtype=torch.float64, device=DEV)
        self.ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
        if keep_host:
            self.h_p, self.h_m, self.h_v = np_f32(self.p), np_f32(self.m), np_f32(self.v)
            self.h_g = [np_bf16(g) for g in self.grads]

    def clone_states(self):
        return self.p.clone(), self.m.clone(), self.v.clone(), torch.zeros_like(self.w)

    def gpu_sqnorm(self, begin=0, end=None, accumulate=False) -> float:
        end = self.n if end is None else end
        gs.gs_grad_sqnorm(self.grads, begin, end, self.sq, self.ws, accumulate=accumulate)
        torch.cuda.synchronize()
        return float(self.sq.item())

    def oracle_step(self, hp: gs.HParams, c: float, begin=0, end=None):
        p, m, v = self.h_p.copy(), self.h_m.copy(), self.h_v.copy()
        w = np.zeros(self.n, np.uint16)
        O.accum_adamw(p, m, v, w, self.h_g, ohp(hp), c, begin, self.n if end is None else end)
        return p, m, v, w

