"""ctypes binding of libgs_mixprobe.so (probe/gs_mixprobe.hip): kernels with the fused step's memory
traffic and no arithmetic, which bench.py times next to gs_accum_adamw.  A measurement aid; the
product path (gs.py / libgs.so) neither imports nor needs it."""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgs_mixprobe.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: run __graft_entry__.build() (or paper_2512_17570_amd.build.build_probe())")

import torch  # noqa: E402,F401  (bind to the HIP runtime PyTorch has loaded)

_lib = ctypes.CDLL(LIB_PATH)
_vp = ctypes.c_void_p
_lib.gs_mixprobe_launch.argtypes = [ctypes.c_int, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                    ctypes.POINTER(_vp), ctypes.c_int, ctypes.c_int64, ctypes.c_uint32, _vp, _vp]
_lib.gs_mixprobe_launch.restype = ctypes.c_int

FUSED_SHALLOW, FUSED_ALL_IN_FLIGHT, READ_HALF, WRITE_HALF = 0, 1, 2, 3


def launch(mode: int, block: int, p, m, v, po, mo, vo, w, grads, n: int, sink, stream) -> None:
    """Enqueue one probe kernel over the first n elements (n a multiple of 4) on `stream`
    (a torch.cuda.Stream).  mask is passed as 0: the values written are the values read."""
    tab = (ctypes.c_void_p * len(grads))(*[g.data_ptr() for g in grads])
    a = [None if t is None else t.data_ptr() for t in (p, m, v, po, mo, vo, w)]
    rc = _lib.gs_mixprobe_launch(mode, block, *a, tab, len(grads), n, 0, sink.data_ptr(), stream.cuda_stream)
    if rc != 0:
        raise RuntimeError(f"gs_mixprobe_launch(mode={mode}, block={block}) failed: {rc}")
