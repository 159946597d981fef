"""Thin ctypes binding of the C ABI in include/gs.h -- argument marshalling only.

Every step of the path runs in the HIP library; this module holds no arithmetic and no
fallback.  Importing it loads ``libgs.so`` (built in-tree by ``paper_2512_17570_amd.build``)
and raises if the library is missing.

Tensors are passed as torch tensors (their device/host address is taken with ``data_ptr()``)
or as raw integer addresses.  Streams are ``torch.cuda.Stream`` objects, raw ``hipStream_t``
integers, or None for torch's current stream.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgs.so")

GS_OK = 0
GS_ERR_INVALID_ARG = -1
GS_ERR_WORKSPACE = -2
GS_ERR_HIP = -3
GS_ERR_NOMEM = -4
GS_ERR_IO = -5
GS_ERR_TOO_LARGE = -6
GS_NOALLOC_MAX_ELEMS = 1 << 33
GS_MAX_K = 32

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build the HIP library first "
        "(python -m paper_2512_17570_amd.build, or __graft_entry__.build()). There is no fallback path.")

# PyTorch owns device memory and streams in this process, so the library must run on the HIP
# runtime PyTorch ships (same SONAME): import torch first so that the dynamic loader binds
# libgs.so to the runtime that is already loaded instead of opening a second one.
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(LIB_PATH)


class gs_adamw_hparams(ctypes.Structure):
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

    def c_struct(self) -> gs_adamw_hparams:
        return gs_adamw_hparams(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay,
                                self.max_grad_norm, self.step)


_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_pp = ctypes.POINTER(ctypes.c_void_p)

_lib.gs_sqnorm_workspace_bytes.argtypes = []
_lib.gs_sqnorm_workspace_bytes.restype = ctypes.c_size_t
_lib.gs_sqnorm_workspace_bytes_for.argtypes = [_i64]
_lib.gs_sqnorm_workspace_bytes_for.restype = ctypes.c_size_t
_lib.gs_grad_sqnorm.argtypes = [_pp, ctypes.c_int, _i64, _i64, _vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp]
_lib.gs_grad_sqnorm.restype = ctypes.c_int
_lib.gs_grad_sqnorm_noalloc.argtypes = [_pp, ctypes.c_int, _i64, _i64, _vp, ctypes.c_int, _vp]
_lib.gs_grad_sqnorm_noalloc.restype = ctypes.c_int
_lib.gs_accum_adamw.argtypes = [_vp, _vp, _vp, _vp, _pp, ctypes.c_int, _i64, _i64,
                                ctypes.POINTER(gs_adamw_hparams), _vp, _vp]
_lib.gs_accum_adamw.restype = ctypes.c_int
_lib.gs_grad_accum_sqnorm.argtypes = [_pp, ctypes.c_int, _i64, _i64, _vp, _vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp]
_lib.gs_grad_accum_sqnorm.restype = ctypes.c_int
_lib.gs_accum_add.argtypes = [_vp, _vp, ctypes.c_int, _i64, _i64, _vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp]
_lib.gs_accum_add.restype = ctypes.c_int
_lib.gs_acc_sqnorm.argtypes = [_vp, _i64, _i64, _vp, ctypes.c_int, _vp, ctypes.c_size_t, _vp]
_lib.gs_acc_sqnorm.restype = ctypes.c_int
_lib.gs_adamw_from_acc.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, ctypes.POINTER(gs_adamw_hparams), _vp, _vp]
_lib.gs_adamw_from_acc.restype = ctypes.c_int
_lib.gs_accum_adamw_oop.argtypes = [_vp] * 7 + [_pp, ctypes.c_int, _i64, _i64, ctypes.POINTER(gs_adamw_hparams), _vp, _vp]
_lib.gs_accum_adamw_oop.restype = ctypes.c_int
_lib.gs_accum_adamw_spec.argtypes = [_vp] * 7 + [_pp, ctypes.c_int, _i64, _i64, ctypes.POINTER(gs_adamw_hparams), _vp,
                                     ctypes.c_int, _vp, ctypes.c_size_t, _vp]
_lib.gs_accum_adamw_spec.restype = ctypes.c_int
_lib.gs_clip_coefficient.argtypes = [ctypes.c_double, ctypes.c_float]
_lib.gs_clip_coefficient.restype = ctypes.c_float
_lib.gs_cu_stream_create.argtypes = [ctypes.POINTER(_vp), ctypes.c_int]
_lib.gs_cu_stream_create.restype = ctypes.c_int
_lib.gs_cu_stream_destroy.argtypes = [_vp]
_lib.gs_cu_stream_destroy.restype = ctypes.c_int
_lib.gs_stream_ctx_create_inplace.argtypes = [ctypes.POINTER(_vp), ctypes.c_int]
_lib.gs_stream_ctx_create.argtypes = [ctypes.POINTER(_vp), _i64, ctypes.c_int]
_lib.gs_stream_ctx_create.restype = ctypes.c_int
_lib.gs_stream_ctx_create_inplace.restype = ctypes.c_int
_lib.gs_stream_ctx_copies_overlap.argtypes = [_vp]
_lib.gs_stream_ctx_copies_overlap.restype = ctypes.c_int
_lib.gs_stream_ctx_destroy.argtypes = [_vp]
_lib.gs_stream_ctx_destroy.restype = ctypes.c_int
_lib.gs_stream_ctx_sync.argtypes = [_vp]
_lib.gs_stream_ctx_sync.restype = ctypes.c_int
_lib.gs_stream_layer_step.argtypes = [_vp, _vp, _vp, _vp, _vp, _pp, ctypes.c_int, _i64,
                                      ctypes.POINTER(gs_adamw_hparams), _vp, _vp]
_lib.gs_stream_layer_step.restype = ctypes.c_int
_lib.gs_pinned_alloc.argtypes = [ctypes.c_size_t]
_lib.gs_pinned_alloc.restype = _vp
_lib.gs_pinned_free.argtypes = [_vp]
_lib.gs_pinned_free.restype = None
_lib.gs_strerror.argtypes = [ctypes.c_int]
_lib.gs_strerror.restype = ctypes.c_char_p
_lib.gs_last_hip_error.argtypes = []
_lib.gs_last_hip_error.restype = ctypes.c_char_p


class GsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {gs_strerror(status)} ({status})"
        if status == GS_ERR_HIP:
            msg += f": {gs_last_hip_error()}"
        super().__init__(msg)


def _addr(x) -> int | None:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(s) -> int | None:
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _need(x, end: int, elem_bytes: int, name: str) -> None:
    """When a tensor (not a raw address) is passed, refuse a range that runs past its end --
    the C ABI sees plain pointers and cannot know."""
    if hasattr(x, "numel"):
        if x.element_size() != elem_bytes:
            raise TypeError(f"{name}: expected {elem_bytes}-byte elements, got {x.dtype}")
        if x.numel() < end:
            raise ValueError(f"{name}: holds {x.numel()} elements, range ends at {end}")
        if not x.is_contiguous():
            raise ValueError(f"{name}: tensor must be contiguous")


def _table(grads):
    addrs = [_addr(g) for g in grads]
    return (ctypes.c_void_p * max(len(addrs), 1))(*addrs), len(addrs)


def _hp(hp):
    if hp is None:
        return None
    return ctypes.byref(hp.c_struct() if isinstance(hp, HParams) else hp)


def _check(status: int, where: str, check: bool) -> int:
    if check and status != GS_OK:
        raise GsError(status, where)
    return status


def gs_strerror(status: int) -> str:
    return _lib.gs_strerror(int(status)).decode()


def gs_last_hip_error() -> str:
    return _lib.gs_last_hip_error().decode()


def gs_sqnorm_workspace_bytes() -> int:
    return int(_lib.gs_sqnorm_workspace_bytes())


def gs_sqnorm_workspace_bytes_for(range_elems: int) -> int:
    return int(_lib.gs_sqnorm_workspace_bytes_for(int(range_elems)))


def gs_grad_sqnorm(grads, begin: int, end: int, d_sqnorm, d_workspace, workspace_bytes: int | None = None,
                   accumulate: bool = False, stream=None, check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size() if hasattr(d_workspace, "numel") else 0
    st = _lib.gs_grad_sqnorm(tab, kk if k is None else k, begin, end, _addr(d_sqnorm), int(bool(accumulate)),
                             _addr(d_workspace), workspace_bytes, _stream(stream))
    return _check(st, "gs_grad_sqnorm", check)


def gs_grad_sqnorm_noalloc(grads, begin: int, end: int, d_sqnorm, accumulate: bool = False, stream=None,
                           check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    st = _lib.gs_grad_sqnorm_noalloc(tab, kk if k is None else k, begin, end, _addr(d_sqnorm), int(bool(accumulate)),
                                     _stream(stream))
    return _check(st, "gs_grad_sqnorm_noalloc", check)


def gs_accum_adamw(p, m, v, w_bf16, grads, begin: int, end: int, hp, d_sqnorm=None, stream=None,
                   check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    for x, eb, nm in ((p, 4, "p"), (m, 4, "m"), (v, 4, "v"), (w_bf16, 2, "w_bf16")):
        _need(x, end, eb, nm)
    st = _lib.gs_accum_adamw(_addr(p), _addr(m), _addr(v), _addr(w_bf16), tab, kk if k is None else k,
                             begin, end, _hp(hp), _addr(d_sqnorm), _stream(stream))
    return _check(st, "gs_accum_adamw", check)


def gs_grad_accum_sqnorm(grads, begin: int, end: int, acc_f32, d_sqnorm, d_workspace,
                         workspace_bytes: int | None = None, accumulate: bool = False, stream=None,
                         check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    _need(acc_f32, end, 4, "acc_f32")
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size() if hasattr(d_workspace, "numel") else 0
    st = _lib.gs_grad_accum_sqnorm(tab, kk if k is None else k, begin, end, _addr(acc_f32), _addr(d_sqnorm),
                                   int(bool(accumulate)), _addr(d_workspace), workspace_bytes, _stream(stream))
    return _check(st, "gs_grad_accum_sqnorm", check)


def gs_accum_add(acc_f32, grad_bf16, first: bool, begin: int, end: int, d_sqnorm=None, d_workspace=None,
                 workspace_bytes: int | None = None, accumulate: bool = False, stream=None,
                 check: bool = True) -> int:
    _need(acc_f32, end, 4, "acc_f32")
    _need(grad_bf16, end, 2, "grad_bf16")
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size() if hasattr(d_workspace, "numel") else 0
    st = _lib.gs_accum_add(_addr(acc_f32), _addr(grad_bf16), int(bool(first)), begin, end, _addr(d_sqnorm),
                           int(bool(accumulate)), _addr(d_workspace), workspace_bytes, _stream(stream))
    return _check(st, "gs_accum_add", check)


def gs_acc_sqnorm(acc_f32, begin: int, end: int, d_sqnorm, d_workspace, workspace_bytes: int | None = None,
                  accumulate: bool = False, stream=None, check: bool = True) -> int:
    _need(acc_f32, end, 4, "acc_f32")
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size() if hasattr(d_workspace, "numel") else 0
    st = _lib.gs_acc_sqnorm(_addr(acc_f32), begin, end, _addr(d_sqnorm), int(bool(accumulate)), _addr(d_workspace),
                            workspace_bytes, _stream(stream))
    return _check(st, "gs_acc_sqnorm", check)


def gs_adamw_from_acc(p, m, v, w_bf16, acc_f32, begin: int, end: int, hp, d_sqnorm=None, stream=None,
                      check: bool = True) -> int:
    for x, eb, nm in ((p, 4, "p"), (m, 4, "m"), (v, 4, "v"), (w_bf16, 2, "w_bf16"), (acc_f32, 4, "acc_f32")):
        _need(x, end, eb, nm)
    st = _lib.gs_adamw_from_acc(_addr(p), _addr(m), _addr(v), _addr(w_bf16), _addr(acc_f32), begin, end,
                                _hp(hp), _addr(d_sqnorm), _stream(stream))
    return _check(st, "gs_adamw_from_acc", check)


def gs_accum_adamw_oop(p, m, v, p_out, m_out, v_out, w_bf16, grads, begin: int, end: int, hp, d_sqnorm=None,
                       stream=None, check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    for x, eb, nm in ((p, 4, "p"), (m, 4, "m"), (v, 4, "v"), (p_out, 4, "p_out"), (m_out, 4, "m_out"),
                      (v_out, 4, "v_out"), (w_bf16, 2, "w_bf16")):
        _need(x, end, eb, nm)
    st = _lib.gs_accum_adamw_oop(_addr(p), _addr(m), _addr(v), _addr(p_out), _addr(m_out), _addr(v_out),
                                 _addr(w_bf16), tab, kk if k is None else k, begin, end, _hp(hp), _addr(d_sqnorm),
                                 _stream(stream))
    return _check(st, "gs_accum_adamw_oop", check)


def gs_accum_adamw_spec(p, m, v, p_out, m_out, v_out, w_bf16, grads, begin: int, end: int, hp, d_sqnorm,
                        d_workspace, workspace_bytes: int | None = None, accumulate: bool = False, stream=None,
                        check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    for x, eb, nm in ((p, 4, "p"), (m, 4, "m"), (v, 4, "v"), (p_out, 4, "p_out"), (m_out, 4, "m_out"),
                      (v_out, 4, "v_out"), (w_bf16, 2, "w_bf16")):
        _need(x, end, eb, nm)
    if workspace_bytes is None:
        workspace_bytes = d_workspace.numel() * d_workspace.element_size() if hasattr(d_workspace, "numel") else 0
    st = _lib.gs_accum_adamw_spec(_addr(p), _addr(m), _addr(v), _addr(p_out), _addr(m_out), _addr(v_out),
                                  _addr(w_bf16), tab, kk if k is None else k, begin, end, _hp(hp), _addr(d_sqnorm),
                                  int(bool(accumulate)), _addr(d_workspace), workspace_bytes, _stream(stream))
    return _check(st, "gs_accum_adamw_spec", check)


def gs_clip_coefficient(sqnorm_total: float, max_grad_norm: float) -> float:
    return float(_lib.gs_clip_coefficient(float(sqnorm_total), float(max_grad_norm)))


def gs_cu_stream_create(num_cus: int, check: bool = True):
    """Returns the raw hipStream_t (int) of a stream confined to `num_cus` compute units."""
    out = ctypes.c_void_p()
    st = _lib.gs_cu_stream_create(ctypes.byref(out), num_cus)
    if check:
        _check(st, "gs_cu_stream_create", True)
        return out.value
    return st, out.value


def gs_cu_stream_destroy(stream, check: bool = True) -> int:
    return _check(_lib.gs_cu_stream_destroy(stream), "gs_cu_stream_destroy", check)


def gs_stream_ctx_create_inplace(num_cus: int = 0, check: bool = True):
    out = ctypes.c_void_p()
    st = _lib.gs_stream_ctx_create_inplace(ctypes.byref(out), num_cus)
    if check:
        _check(st, "gs_stream_ctx_create_inplace", True)
        return out.value
    return st, out.value


def gs_stream_ctx_create(chunk_elems: int, slots: int = 3, check: bool = True):
    out = ctypes.c_void_p()
    st = _lib.gs_stream_ctx_create(ctypes.byref(out), chunk_elems, slots)
    if check:
        _check(st, "gs_stream_ctx_create", True)
        return out.value
    return st, out.value


def gs_stream_ctx_copies_overlap(ctx) -> int:
    return int(_lib.gs_stream_ctx_copies_overlap(ctx))


def gs_stream_ctx_destroy(ctx, check: bool = True) -> int:
    return _check(_lib.gs_stream_ctx_destroy(ctx), "gs_stream_ctx_destroy", check)


def gs_stream_ctx_sync(ctx, check: bool = True) -> int:
    return _check(_lib.gs_stream_ctx_sync(ctx), "gs_stream_ctx_sync", check)


def gs_stream_layer_step(ctx, h_p, h_m, h_v, d_w_bf16, d_grads, n: int, hp, d_sqnorm=None,
                         producer_stream=None, check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(d_grads) if d_grads is not None else (None, 0)
    for j, g in enumerate(d_grads or ()):
        _need(g, n, 2, f"d_grads[{j}]")
    for x, eb, nm in ((h_p, 4, "h_p"), (h_m, 4, "h_m"), (h_v, 4, "h_v"), (d_w_bf16, 2, "d_w_bf16")):
        _need(x, n, eb, nm)
    st = _lib.gs_stream_layer_step(ctx, _addr(h_p), _addr(h_m), _addr(h_v), _addr(d_w_bf16), tab,
                                   kk if k is None else k, n, _hp(hp), _addr(d_sqnorm), _stream(producer_stream))
    return _check(st, "gs_stream_layer_step", check)


class gs_tier_layer(ctypes.Structure):
    _fields_ = [("h_p", ctypes.c_void_p), ("h_m", ctypes.c_void_p), ("h_v", ctypes.c_void_p),
                ("n_host", ctypes.c_int64),
                ("fd_p", ctypes.c_int), ("fd_m", ctypes.c_int), ("fd_v", ctypes.c_int),
                ("off_p", ctypes.c_int64), ("off_m", ctypes.c_int64), ("off_v", ctypes.c_int64)]


_lib.gs_tier_ctx_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), _i64, ctypes.c_int, ctypes.c_int]
_lib.gs_tier_ctx_create.restype = ctypes.c_int
_lib.gs_tier_ctx_destroy.argtypes = [_vp]
_lib.gs_tier_ctx_destroy.restype = ctypes.c_int
_lib.gs_tier_ctx_sync.argtypes = [_vp]
_lib.gs_tier_ctx_sync.restype = ctypes.c_int
_lib.gs_tier_ctx_error.argtypes = [_vp]
_lib.gs_tier_ctx_error.restype = ctypes.c_char_p
_lib.gs_tier_layer_step.argtypes = [_vp, ctypes.POINTER(gs_tier_layer), _vp, _pp, ctypes.c_int, _i64, _vp, _vp, _vp]
_lib.gs_tier_layer_step.restype = ctypes.c_int


def gs_tier_ctx_create(chunk_elems: int, slots: int = 3, num_cus: int = 0, check: bool = True):
    out = ctypes.c_void_p()
    st = _lib.gs_tier_ctx_create(ctypes.byref(out), chunk_elems, slots, num_cus)
    if check:
        _check(st, "gs_tier_ctx_create", True)
        return out.value
    return st, out.value


def gs_tier_ctx_destroy(ctx, check: bool = True) -> int:
    return _check(_lib.gs_tier_ctx_destroy(ctx), "gs_tier_ctx_destroy", check)


def gs_tier_ctx_sync(ctx, check: bool = True) -> int:
    return _check(_lib.gs_tier_ctx_sync(ctx), "gs_tier_ctx_sync", check)


def gs_tier_ctx_error(ctx) -> str:
    return (_lib.gs_tier_ctx_error(ctx) or b"").decode()


def gs_tier_layer_step(ctx, h_p, h_m, h_v, n_host: int, fds, offsets, d_w_bf16, d_grads, n: int, hp,
                       d_sqnorm=None, producer_stream=None, check: bool = True, k: int | None = None,
                       layer: "gs_tier_layer | None" = None) -> int:
    """fds = (fd_p, fd_m, fd_v) and offsets = (off_p, off_m, off_v) in bytes; `layer` passes a
    ready-made descriptor (or None with check=False to exercise the rejection).  The call queues
    the layer and returns: keep the tensors alive and untouched until gs_tier_ctx_sync, which also
    reports I/O failures."""
    tab, kk = _table(d_grads) if d_grads is not None else (None, 0)
    for j, g in enumerate(d_grads or ()):
        _need(g, n, 2, f"d_grads[{j}]")
    _need(d_w_bf16, n, 2, "d_w_bf16")
    if layer is None and fds is not None:
        for x, nm in ((h_p, "h_p"), (h_m, "h_m"), (h_v, "h_v")):
            _need(x, n_host, 4, nm)
        layer = gs_tier_layer(_addr(h_p), _addr(h_m), _addr(h_v), n_host, fds[0], fds[1], fds[2],
                              offsets[0], offsets[1], offsets[2])
    st = _lib.gs_tier_layer_step(ctx, ctypes.byref(layer) if layer is not None else None, _addr(d_w_bf16), tab,
                                 kk if k is None else k, n, _hp(hp), _addr(d_sqnorm), _stream(producer_stream))
    return _check(st, "gs_tier_layer_step", check)


_lib.gs_stream_layer_step_range.argtypes = [_vp, _vp, _vp, _vp, _vp, _pp, ctypes.c_int, _i64, _i64, _vp, _vp, _vp]
_lib.gs_stream_layer_step_range.restype = ctypes.c_int
_lib.gs_tier_layer_step_range.argtypes = [_vp, ctypes.POINTER(gs_tier_layer), _vp, _pp, ctypes.c_int, _i64, _i64, _i64,
                                          _vp, _vp, _vp]
_lib.gs_tier_layer_step_range.restype = ctypes.c_int


def gs_stream_layer_step_range(ctx, h_p, h_m, h_v, d_w_bf16, d_grads, begin: int, end: int, hp, d_sqnorm=None,
                               producer_stream=None, check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(d_grads) if d_grads is not None else (None, 0)
    for j, g in enumerate(d_grads or ()):
        _need(g, end, 2, f"d_grads[{j}]")
    for x, eb, nm in ((h_p, 4, "h_p"), (h_m, 4, "h_m"), (h_v, 4, "h_v"), (d_w_bf16, 2, "d_w_bf16")):
        _need(x, end, eb, nm)
    st = _lib.gs_stream_layer_step_range(ctx, _addr(h_p), _addr(h_m), _addr(h_v), _addr(d_w_bf16), tab,
                                         kk if k is None else k, begin, end, _hp(hp), _addr(d_sqnorm),
                                         _stream(producer_stream))
    return _check(st, "gs_stream_layer_step_range", check)


def gs_tier_layer_step_range(ctx, h_p, h_m, h_v, n_host: int, fds, offsets, d_w_bf16, d_grads, n: int, begin: int,
                             end: int, hp, d_sqnorm=None, producer_stream=None, check: bool = True,
                             k: int | None = None) -> int:
    tab, kk = _table(d_grads) if d_grads is not None else (None, 0)
    for j, g in enumerate(d_grads or ()):
        _need(g, n, 2, f"d_grads[{j}]")
    _need(d_w_bf16, n, 2, "d_w_bf16")
    for x, nm in ((h_p, "h_p"), (h_m, "h_m"), (h_v, "h_v")):
        _need(x, n_host, 4, nm)
    layer = gs_tier_layer(_addr(h_p), _addr(h_m), _addr(h_v), n_host, fds[0], fds[1], fds[2],
                          offsets[0], offsets[1], offsets[2])
    st = _lib.gs_tier_layer_step_range(ctx, ctypes.byref(layer), _addr(d_w_bf16), tab, kk if k is None else k, n,
                                       begin, end, _hp(hp), _addr(d_sqnorm), _stream(producer_stream))
    return _check(st, "gs_tier_layer_step_range", check)


def gs_pinned_alloc(nbytes: int) -> int | None:
    return _lib.gs_pinned_alloc(nbytes)


def gs_pinned_free(ptr) -> None:
    _lib.gs_pinned_free(ptr)


def pinned_f32(n: int):
    """A float32 torch tensor over n elements of memory from gs_pinned_alloc.  Returns
    (tensor, ptr); the caller frees ptr with gs_pinned_free after dropping the tensor."""
    import numpy as np
    import torch
    ptr = gs_pinned_alloc(n * 4)
    if not ptr:
        raise MemoryError(f"gs_pinned_alloc({n * 4}) failed: {gs_last_hip_error()}")
    buf = (ctypes.c_float * n).from_address(ptr)
    return torch.from_numpy(np.ctypeslib.as_array(buf)), ptr


def pinned_f32_set(n: int, count: int = 3):
    """`count` pinned float32 tensors of n elements each, or None if the host cannot pin that much
    (anything allocated on the way is released).  Returns [(tensor, ptr), ...]."""
    got = []
    try:
        for _ in range(count):
            got.append(pinned_f32(n))
        return got
    except MemoryError:
        for _, ptr in got:
            gs_pinned_free(ptr)
        return None


_lib.gs_defer_ctx_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int]
_lib.gs_defer_ctx_create.restype = ctypes.c_int
_lib.gs_defer_ctx_destroy.argtypes = [_vp]
_lib.gs_defer_ctx_destroy.restype = ctypes.c_int
_lib.gs_defer_ctx_sync.argtypes = [_vp]
_lib.gs_defer_ctx_sync.restype = ctypes.c_int
_lib.gs_defer_layer_step.argtypes = [_vp, ctypes.c_int, _vp, _vp, _vp, _vp, _pp, ctypes.c_int, _i64, _i64,
                                     ctypes.POINTER(gs_adamw_hparams), _vp, _vp]
_lib.gs_defer_layer_step.restype = ctypes.c_int
_lib.gs_defer_wait_layer.argtypes = [_vp, ctypes.c_int, _vp]
_lib.gs_defer_wait_layer.restype = ctypes.c_int
_lib.gs_defer_layer_done.argtypes = [_vp, ctypes.c_int]
_lib.gs_defer_layer_done.restype = ctypes.c_int


def gs_defer_ctx_create(max_layers: int, num_cus: int = 0, check: bool = True):
    out = ctypes.c_void_p()
    st = _lib.gs_defer_ctx_create(ctypes.byref(out), max_layers, num_cus)
    if check:
        _check(st, "gs_defer_ctx_create", True)
        return out.value
    return st, out.value


_lib.gs_defer_ctx_stream.argtypes = [_vp]
_lib.gs_defer_ctx_stream.restype = _vp


def gs_defer_ctx_stream(ctx) -> int | None:
    """Raw hipStream_t of the context's stream (owned by the context)."""
    return _lib.gs_defer_ctx_stream(ctx)


def gs_defer_ctx_destroy(ctx, check: bool = True) -> int:
    return _check(_lib.gs_defer_ctx_destroy(ctx), "gs_defer_ctx_destroy", check)


def gs_defer_ctx_sync(ctx, check: bool = True) -> int:
    return _check(_lib.gs_defer_ctx_sync(ctx), "gs_defer_ctx_sync", check)


def gs_defer_layer_step(ctx, layer: int, p, m, v, w_bf16, grads, begin: int, end: int, hp, d_sqnorm=None,
                        producer_stream=None, check: bool = True, k: int | None = None) -> int:
    tab, kk = _table(grads) if grads is not None else (None, 0)
    for j, g in enumerate(grads or ()):
        _need(g, end, 2, f"grads[{j}]")
    for x, eb, nm in ((p, 4, "p"), (m, 4, "m"), (v, 4, "v"), (w_bf16, 2, "w_bf16")):
        _need(x, end, eb, nm)
    st = _lib.gs_defer_layer_step(ctx, layer, _addr(p), _addr(m), _addr(v), _addr(w_bf16), tab, kk if k is None else k,
                                  begin, end, _hp(hp), _addr(d_sqnorm), _stream(producer_stream))
    return _check(st, "gs_defer_layer_step", check)


def gs_defer_wait_layer(ctx, layer: int, consumer_stream=None, check: bool = True) -> int:
    return _check(_lib.gs_defer_wait_layer(ctx, layer, _stream(consumer_stream)), "gs_defer_wait_layer", check)


def gs_defer_layer_done(ctx, layer: int) -> int:
    return int(_lib.gs_defer_layer_done(ctx, layer))
