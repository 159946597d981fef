"""ctypes loader for the scalar C oracle (``gs_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by ``__graft_entry__.smoke()`` and by the
benchmark's ``cpu_baseline`` leg.  The product path (the HIP library and its Python binding)
never imports this module and shares no code with it.

All arrays are numpy: fp32 states as ``float32``, bf16 tensors as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gs_oracle.c")
_LIB = os.path.join(_HERE, "libgs_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = f"{_LIB}.{os.getpid()}.tmp"       # written aside, then renamed: parallel test workers may build at once
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-Wall", "-Wextra",
               "-shared", "-fPIC", _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _HP(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("max_grad_norm", ctypes.c_float), ("step", ctypes.c_int32)]


@dataclass
class HParams:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    max_grad_norm: float = 1.0
    step: int = 1

    def _c(self) -> _HP:
        return _HP(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay,
                   self.max_grad_norm, self.step)


_lib = None


def lib():
    global _lib
    if _lib is None:
        # GS_ORACLE_LIB: used only by the mutation test, which points the pins at a deliberately
        # broken build of the oracle to show that they notice.
        L = ctypes.CDLL(os.environ.get("GS_ORACLE_LIB") or build())
        u16pp = ctypes.POINTER(ctypes.c_void_p)
        L.gs_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.gs_oracle_bf16_to_f32.restype = ctypes.c_float
        L.gs_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.gs_oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.gs_oracle_grad_sqnorm.argtypes = [u16pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64]
        L.gs_oracle_grad_sqnorm.restype = ctypes.c_double
        L.gs_oracle_accumulate.argtypes = [u16pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        L.gs_oracle_accumulate.restype = None
        L.gs_oracle_accum_add.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64]
        L.gs_oracle_accum_add.restype = ctypes.c_double
        L.gs_oracle_acc_sqnorm.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64]
        L.gs_oracle_acc_sqnorm.restype = ctypes.c_double
        L.gs_oracle_clip_coef.argtypes = [ctypes.c_double, ctypes.c_float]
        L.gs_oracle_clip_coef.restype = ctypes.c_float
        L.gs_oracle_accum_adamw.argtypes = [ctypes.c_void_p] * 4 + [
            u16pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(_HP), ctypes.c_float]
        L.gs_oracle_accum_adamw.restype = None
        L.gs_oracle_accum_adamw_f64.argtypes = [ctypes.c_void_p] * 6 + [
            u16pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(_HP), ctypes.c_double]
        L.gs_oracle_accum_adamw_f64.restype = None
        _lib = L
    return _lib


def _check(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags.c_contiguous or a.ndim != 1:
        raise TypeError(f"{name}: need contiguous 1-D numpy array of {np.dtype(dtype)}")
    return a


def _grad_table(grads):
    gs = [_check(g, np.uint16, "grad") for g in grads]
    n = len(gs[0])
    if any(len(g) != n for g in gs):
        raise ValueError("gradient buffers differ in length")
    tab = (ctypes.c_void_p * len(gs))(*[g.ctypes.data for g in gs])
    return tab, len(gs), n


def bf16_to_f32(h: int) -> float:
    return float(lib().gs_oracle_bf16_to_f32(int(h) & 0xFFFF))


def f32_to_bf16(x) -> int:
    return int(lib().gs_oracle_f32_to_bf16(np.float32(x)))


def grad_sqnorm(grads, begin: int = 0, end: int | None = None) -> float:
    """Squared L2 norm of the fp32 sum of the k bf16 buffers over [begin,end)."""
    tab, k, n = _grad_table(grads)
    end = n if end is None else end
    assert 0 <= begin <= end <= n
    return float(lib().gs_oracle_grad_sqnorm(tab, k, begin, end))


def accumulate(grads, begin: int = 0, end: int | None = None) -> np.ndarray:
    """fp32 sum of the k bf16 buffers (j ascending); entries outside [begin,end) are 0."""
    tab, k, n = _grad_table(grads)
    end = n if end is None else end
    assert 0 <= begin <= end <= n
    out = np.zeros(n, np.float32)
    lib().gs_oracle_accumulate(tab, k, begin, end, out.ctypes.data)
    return out


def accum_add(acc: np.ndarray, grad: np.ndarray, first: bool, begin: int = 0, end: int | None = None) -> float:
    """acc[i] = (first ? +0 : acc[i]) + grad[i] over [begin,end), in place; returns the squared
    L2 norm of the updated range."""
    _check(acc, np.float32, "acc")
    _check(grad, np.uint16, "grad")
    end = len(grad) if end is None else end
    assert 0 <= begin <= end <= len(grad) and len(acc) >= end
    return float(lib().gs_oracle_accum_add(acc.ctypes.data, grad.ctypes.data, int(bool(first)), begin, end))


def acc_sqnorm(acc: np.ndarray, begin: int = 0, end: int | None = None) -> float:
    """Squared L2 norm of a finished fp32 accumulation buffer over [begin,end)."""
    _check(acc, np.float32, "acc")
    end = len(acc) if end is None else end
    assert 0 <= begin <= end <= len(acc)
    return float(lib().gs_oracle_acc_sqnorm(acc.ctypes.data, begin, end))


def clip_coef(sqnorm_total: float, max_norm: float) -> float:
    return float(lib().gs_oracle_clip_coef(float(sqnorm_total), np.float32(max_norm)))


def accum_adamw(p, m, v, w, grads, hp: HParams, c: float = 1.0,
                begin: int = 0, end: int | None = None) -> None:
    """fp32 reference-order step over [begin,end); p, m, v updated in place, w written."""
    tab, k, n = _grad_table(grads)
    end = n if end is None else end
    assert 0 <= begin <= end <= n
    for a, dt, nm in ((p, np.float32, "p"), (m, np.float32, "m"), (v, np.float32, "v"), (w, np.uint16, "w")):
        _check(a, dt, nm)
        assert len(a) >= end
    hpc = hp._c()
    lib().gs_oracle_accum_adamw(p.ctypes.data, m.ctypes.data, v.ctypes.data, w.ctypes.data,
                                tab, k, begin, end, ctypes.byref(hpc), np.float32(c))


def accum_adamw_f64(p, m, v, grads, hp: HParams, sqnorm_total: float = -1.0,
                    begin: int = 0, end: int | None = None):
    """Double-precision evaluation of the same step; returns (p', m', v') as float64 arrays
    (entries outside [begin,end) are NaN).  ``sqnorm_total < 0`` means no clipping."""
    tab, k, n = _grad_table(grads)
    end = n if end is None else end
    assert 0 <= begin <= end <= n
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _check(a, np.float32, nm)
    po = np.full(n, np.nan); mo = np.full(n, np.nan); vo = np.full(n, np.nan)
    hpc = hp._c()
    lib().gs_oracle_accum_adamw_f64(p.ctypes.data, m.ctypes.data, v.ctypes.data,
                                    po.ctypes.data, mo.ctypes.data, vo.ctypes.data,
                                    tab, k, begin, end, ctypes.byref(hpc), float(sqnorm_total))
    return po, mo, vo
