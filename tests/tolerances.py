"""Tolerance readings shared by the CPU pins and the GPU parity tests (no GPU, no library needed)."""
import numpy as np


def f64_truth_check(got: np.ndarray, truth: np.ndarray, old: np.ndarray, name: str):
    """fp32 result against the fp64 evaluation of the same formulas (the arbiter between oracle
    and kernel).  Reading of the tolerance: the stated bound -- 4 fp32 ulp of the result or 1e-6
    relative -- is asserted wherever the final add of the update does not cancel, i.e. where the
    result is at least half as large as its larger operand (|old state|, or the increment
    |new - old|).  Where it cancels (p*decay - step, beta1*m + (1-beta1)*g with opposite signs)
    a bound in units of the result is not meaningful for a chain of ~10 fp32 roundings, and the
    error is held to 8 fp32 spacings of the larger operand instead.  Returns the share of elements
    judged by the stated bound and the worst errors under both bounds."""
    got64 = got.astype(np.float64)
    err = np.abs(got64 - truth)
    t32 = np.abs(truth).astype(np.float32)
    scale = np.maximum(t32, np.maximum(np.abs(old), np.abs(truth - old).astype(np.float32)))
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(err == 0.0, 0.0, err / np.abs(truth))
    stated_ok = (err <= 4.0 * np.spacing(t32).astype(np.float64)) | (rel <= 1e-6)
    operand_ok = err <= 8.0 * np.spacing(scale).astype(np.float64)
    plain = t32 >= 0.5 * scale                     # no cancellation in the final add
    bad_plain = plain & ~stated_ok
    assert not bad_plain.any(), (f"{name}: {int(bad_plain.sum())} non-cancelling elements beyond 4 ulp / 1e-6 of the "
                                 f"fp64 result, worst rel {float(rel[bad_plain].max()):.3e}")
    bad_rest = ~plain & ~(stated_ok | operand_ok)
    assert not bad_rest.any(), f"{name}: {int(bad_rest.sum())} cancelling elements beyond 8 spacings of the larger operand"
    return float(plain.mean()), float(rel[plain].max()) if plain.any() else 0.0, \
        float((err / np.spacing(scale).astype(np.float64)).max())
