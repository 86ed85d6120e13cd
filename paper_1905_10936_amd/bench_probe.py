"""Python binding of libef_bench (include/ef_bench.h): the bandwidth probes bench.py runs beside the
library.  Argument marshalling only; not part of the hot path."""
import ctypes
import os

import torch

from . import EfError, _ptr, _stream_ptr, ef_strerror
from . import build as _build

BENCH_SYMBOLS = ("ef_stream_probe", "ef_stream_probe_grouped")

_lib = None


def lib():
    """Load libef_bench.so (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.BENCH_LIB):
            _build.build(force=True, lib=_build.BENCH_LIB)
        L = ctypes.CDLL(_build.BENCH_LIB)
        vp, i64, c_int, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        L.ef_stream_probe.restype = c_int
        L.ef_stream_probe.argtypes = [vp, vp, vp, i64, c_int, ctypes.POINTER(f32), vp]
        L.ef_stream_probe_grouped.restype = c_int
        L.ef_stream_probe_grouped.argtypes = [vp, vp, vp, i64, c_int, c_int, ctypes.POINTER(f32), vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise EfError(rc, ef_strerror(rc))


def _same_length(g, m, e):
    n = g.numel()
    if m.numel() != n or e.numel() != n:
        raise TypeError("g, m, e must have the same number of elements")
    return n


def ef_stream_probe(g, m, e, repeats=5, stream=None):
    """Bare 3-read/2-write stream over the whole tiles of g, m, e (1-D float32, same length; m and e
    are overwritten with garbage).  Returns (ms per pass, bytes per pass)."""
    n = _same_length(g, m, e)
    ms = ctypes.c_float(0.0)
    _check(lib().ef_stream_probe(_ptr(g, torch.float32, "g"), _ptr(m, torch.float32, "m"),
                                 _ptr(e, torch.float32, "e"), n, int(repeats), ctypes.byref(ms), _stream_ptr(stream)))
    return float(ms.value), 20 * (n // 4096) * 4096


def ef_stream_probe_grouped(g, m, e, group=16, repeats=5, stream=None):
    """As ef_stream_probe, one workgroup per tile, e written in step by groups of `group` tiles."""
    n = _same_length(g, m, e)
    ms = ctypes.c_float(0.0)
    _check(lib().ef_stream_probe_grouped(_ptr(g, torch.float32, "g"), _ptr(m, torch.float32, "m"),
                                         _ptr(e, torch.float32, "e"), n, int(group), int(repeats), ctypes.byref(ms),
                                         _stream_ptr(stream)))
    return float(ms.value), 20 * (n // 4096) * 4096
