"""Python binding of libef (include/ef.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI; this module
turns torch tensors into device pointers and raises on error codes.  There is
no CPU fallback: if libef.so is missing or cannot be loaded, importing the
entry points fails loudly.

Names follow the C ABI: ef_plan_create / ef_worker_step / ef_server_step /
ef_apply (Algorithm 4 of arxiv 1905.10936).
"""
import ctypes
import os

import numpy as np
import torch

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libef.so")

EF_OK, EF_ERR_NULL, EF_ERR_OFFSETS, EF_ERR_ARG, EF_ERR_ALIGN, EF_ERR_HIP, EF_ERR_SIZE = 0, -1, -2, -3, -4, -5, -6
EF_MAX_WORKERS = 64

# what include/ef.h declares (the boundary of Algorithm 4) ...
ABI_SYMBOLS = (
    "ef_plan_create", "ef_plan_destroy", "ef_plan_d", "ef_plan_blocks", "ef_sign_words",
    "ef_worker_step", "ef_server_step", "ef_apply", "ef_strerror",
    "ef_worker_step_sgd", "ef_apply_wd",
    "ef_payload_bytes", "ef_payload_scales_offset", "ef_worker_step_fused", "ef_server_step_fused", "ef_apply_fused",
    "ef_compressor_quality", "ef_compressor_quality_static", "ef_worker_step_quality",
    "ef_plan_set_lazy", "ef_plan_is_lazy", "ef_flush",
    "ef_state_create", "ef_state_destroy", "ef_worker_step_state", "ef_server_step_state", "ef_state_export",
    "ef_state_import",
)
# ... and what include/ef_debug.h declares (tuning and diagnostics the tests use)
DEBUG_SYMBOLS = (
    "ef_plan_tune", "ef_plan_fuse_limit", "ef_plan_set_persistent", "ef_plan_is_persistent", "ef_plan_set_sync_group",
    "ef_plan_last_fallbacks",
)


class EfError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libef error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """Load libef.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        _build.build(force=True, lib=LIB_PATH)
    elif _build.stale(LIB_PATH):
        import warnings
        warnings.warn("libef.so is older than its sources: run paper_1905_10936_amd/build.py", RuntimeWarning)
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, c_int, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    L.ef_plan_create.restype = c_int
    L.ef_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(i64), i64, c_int, vp]
    L.ef_plan_destroy.restype = c_int
    L.ef_plan_destroy.argtypes = [vp]
    for name in ("ef_plan_d", "ef_plan_blocks"):
        getattr(L, name).restype = i64
        getattr(L, name).argtypes = [vp]
    L.ef_sign_words.restype = ctypes.c_size_t
    L.ef_sign_words.argtypes = [vp]
    L.ef_plan_tune.restype = c_int
    L.ef_plan_tune.argtypes = [vp, c_int, c_int]
    L.ef_plan_set_persistent.restype = c_int
    L.ef_plan_set_persistent.argtypes = [vp, c_int]
    L.ef_plan_is_persistent.restype = c_int
    L.ef_plan_is_persistent.argtypes = [vp]
    L.ef_plan_set_lazy.restype = c_int
    L.ef_plan_set_lazy.argtypes = [vp, c_int]
    L.ef_plan_set_sync_group.restype = c_int
    L.ef_plan_set_sync_group.argtypes = [vp, c_int]
    L.ef_plan_is_lazy.restype = c_int
    L.ef_plan_is_lazy.argtypes = [vp]
    L.ef_flush.restype = c_int
    L.ef_flush.argtypes = [vp, c_int, vp, i64, vp, vp]
    L.ef_plan_last_fallbacks.restype = c_int
    L.ef_plan_last_fallbacks.argtypes = [vp, ctypes.POINTER(ctypes.c_uint), ctypes.POINTER(ctypes.c_uint)]
    L.ef_plan_fuse_limit.restype = c_int
    L.ef_plan_fuse_limit.argtypes = [vp]
    L.ef_worker_step.restype = c_int
    L.ef_worker_step.argtypes = [vp, c_int, vp, i64, vp, vp, i64, f32, f32, f32, vp, vp, vp]
    L.ef_worker_step_quality.restype = c_int
    L.ef_worker_step_quality.argtypes = [vp, c_int, vp, i64, vp, vp, i64, f32, f32, f32, vp, vp, vp, vp]
    L.ef_worker_step_sgd.restype = c_int
    L.ef_worker_step_sgd.argtypes = [vp, c_int, vp, i64, vp, i64, f32, f32, vp, vp, vp]
    L.ef_server_step.restype = c_int
    L.ef_server_step.argtypes = [vp, c_int, vp, vp, vp, f32, f32, vp, vp, vp]
    L.ef_apply.restype = c_int
    L.ef_apply.argtypes = [vp, vp, vp, vp, f32, vp]
    L.ef_payload_bytes.restype = ctypes.c_size_t
    L.ef_payload_bytes.argtypes = [vp]
    L.ef_payload_scales_offset.restype = ctypes.c_size_t
    L.ef_payload_scales_offset.argtypes = [vp]
    L.ef_worker_step_fused.restype = c_int
    L.ef_worker_step_fused.argtypes = [vp, c_int, vp, i64, vp, vp, i64, f32, f32, f32, vp, vp]
    L.ef_server_step_fused.restype = c_int
    L.ef_server_step_fused.argtypes = [vp, c_int, vp, vp, f32, f32, vp, vp]
    L.ef_apply_fused.restype = c_int
    L.ef_apply_fused.argtypes = [vp, vp, vp, f32, vp]
    for name in ("ef_compressor_quality", "ef_compressor_quality_static"):
        getattr(L, name).restype = c_int
        getattr(L, name).argtypes = [vp, c_int, vp, i64, vp, vp]
    L.ef_apply_wd.restype = c_int
    L.ef_apply_wd.argtypes = [vp, vp, vp, vp, vp, f32, f32, f32, vp]
    L.ef_state_create.restype = c_int
    L.ef_state_create.argtypes = [vp, c_int, ctypes.POINTER(vp), vp]
    L.ef_state_destroy.restype = c_int
    L.ef_state_destroy.argtypes = [vp]
    L.ef_worker_step_state.restype = c_int
    L.ef_worker_step_state.argtypes = [vp, vp, vp, i64, f32, f32, f32, vp, vp, vp]
    L.ef_server_step_state.restype = c_int
    L.ef_server_step_state.argtypes = [vp, vp, c_int, vp, vp, f32, f32, vp, vp, vp]
    for name in ("ef_state_export", "ef_state_import"):
        getattr(L, name).restype = c_int
        getattr(L, name).argtypes = [vp, vp, vp, vp, i64, vp, vp]
    L.ef_strerror.restype = ctypes.c_char_p
    L.ef_strerror.argtypes = [c_int]
    _lib = L
    return L


def ef_strerror(code):
    return lib().ef_strerror(int(code)).decode()


def _check(rc):
    if rc != EF_OK:
        raise EfError(rc, ef_strerror(rc))


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA/HIP torch tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stride(t, d, name):
    """Row stride in elements of a [n][d'] (or [d']) tensor holding rows of d."""
    if t.dim() == 1:
        return t.numel()
    if t.dim() != 2:
        raise TypeError("%s must be 1-D or 2-D" % name)
    return t.stride(0)


def ef_sign_words(plan):
    return int(lib().ef_sign_words(plan._h))


class Plan:
    """ef_plan: the per-layout object of the C ABI (block partition of
    Section 3.2 + scratch).  Use on the device that was current at creation."""

    def __init__(self, block_offsets, max_workers, stream=None):
        offs = np.ascontiguousarray(block_offsets, dtype=np.int64)
        if offs.ndim != 1 or offs.size < 2:
            raise EfError(EF_ERR_OFFSETS, "block_offsets must hold B+1 >= 2 entries")
        self._h = ctypes.c_void_p()
        rc = lib().ef_plan_create(ctypes.byref(self._h), offs.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                  offs.size - 1, int(max_workers), None)
        _check(rc)
        self.d = int(lib().ef_plan_d(self._h))
        self.B = int(lib().ef_plan_blocks(self._h))
        self.W = int(lib().ef_sign_words(self._h))
        self.max_workers = int(max_workers)

    def tune(self, fuse_limit=-1, spin_limit=-1):
        _check(lib().ef_plan_tune(self._h, int(fuse_limit), int(spin_limit)))

    def set_persistent(self, on):
        """True/False, or None for the choice made at plan creation."""
        _check(lib().ef_plan_set_persistent(self._h, -1 if on is None else int(bool(on))))

    @property
    def persistent(self):
        return bool(lib().ef_plan_is_persistent(self._h))

    def set_lazy(self, on):
        """Deferred residual correction for blocks larger than fuse_limit (see ef_plan_set_lazy)."""
        _check(lib().ef_plan_set_lazy(self._h, int(bool(on))))

    def set_sync_group(self, tiles):
        """Tiles of a large block that are written out in step (0 or 1: off)."""
        _check(lib().ef_plan_set_sync_group(self._h, int(tiles)))

    @property
    def lazy(self):
        return bool(lib().ef_plan_is_lazy(self._h))

    def last_fallbacks(self):
        """(parked_tiles, late_blocks) of the most recent worker/server call."""
        a, b = ctypes.c_uint(0), ctypes.c_uint(0)
        _check(lib().ef_plan_last_fallbacks(self._h, ctypes.byref(a), ctypes.byref(b)))
        return int(a.value), int(b.value)

    @property
    def fuse_limit(self):
        return int(lib().ef_plan_fuse_limit(self._h))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().ef_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ef_plan_create(block_offsets, max_workers, stream=None):
    return Plan(block_offsets, max_workers, stream)


def ef_flush(plan, err=None, server_err=None, stream=None):
    """Writes the deferred corrections into err ([n][>=d] or [d], or None) and server_err ([d], or None)."""
    n, ss, ep = 1, plan.d, None
    if err is not None:
        n = 1 if err.dim() == 1 else err.shape[0]
        ss = _stride(err, plan.d, "err")
        ep = _ptr(err, torch.float32, "err")
    sp = None
    if server_err is not None:
        if server_err.numel() != plan.d:
            raise TypeError("server_err must hold d entries")
        sp = _ptr(server_err, torch.float32, "server_err")
    _check(lib().ef_flush(plan._h, n, ep, ss, sp, _stream_ptr(stream)))


def ef_plan_destroy(plan):
    plan.close()


def ef_worker_step(plan, grad, mom, err, mu, eta_prev, eta, packed_signs, scales, stream=None):
    """grad/mom/err: float32 [n][>=d] (or [d]); packed_signs int64|uint64 [n][W];
    scales float32 [n][B].  mom, err, packed_signs, scales are written."""
    n = 1 if grad.dim() == 1 else grad.shape[0]
    gs, ss = _stride(grad, plan.d, "grad"), _stride(mom, plan.d, "mom")
    if _stride(err, plan.d, "err") != ss or mom.shape != err.shape:
        raise TypeError("mom and err must share shape and stride")
    if packed_signs.numel() != n * plan.W or scales.numel() != n * plan.B:
        raise TypeError("packed_signs must hold n*W words and scales n*B floats")
    rc = lib().ef_worker_step(plan._h, n, _ptr(grad, torch.float32, "grad"), gs,
                              _ptr(mom, torch.float32, "mom"), _ptr(err, torch.float32, "err"), ss,
                              float(mu), float(eta_prev), float(eta),
                              _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                              _ptr(scales, torch.float32, "scales"), _stream_ptr(stream))
    _check(rc)


def ef_worker_step_quality(plan, grad, mom, err, mu, eta_prev, eta, packed_signs, scales, quality, stream=None):
    """ef_worker_step that also writes (phi(p_i), delta(p_i)) of every worker's corrected gradient
    into quality: float64 [n][2]."""
    n = 1 if grad.dim() == 1 else grad.shape[0]
    gs, ss = _stride(grad, plan.d, "grad"), _stride(mom, plan.d, "mom")
    if _stride(err, plan.d, "err") != ss or mom.shape != err.shape:
        raise TypeError("mom and err must share shape and stride")
    if packed_signs.numel() != n * plan.W or scales.numel() != n * plan.B or quality.numel() != 2 * n:
        raise TypeError("packed_signs must hold n*W words, scales n*B floats, quality 2*n doubles")
    rc = lib().ef_worker_step_quality(plan._h, n, _ptr(grad, torch.float32, "grad"), gs,
                                      _ptr(mom, torch.float32, "mom"), _ptr(err, torch.float32, "err"), ss,
                                      float(mu), float(eta_prev), float(eta),
                                      _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                                      _ptr(scales, torch.float32, "scales"), _ptr(quality, torch.float64, "quality"),
                                      _stream_ptr(stream))
    _check(rc)


def ef_server_step(plan, M, packed_signs, scales, server_err, eta_prev, eta, out_signs, out_scales,
                   stream=None):
    if packed_signs.numel() != M * plan.W or scales.numel() != M * plan.B:
        raise TypeError("packed_signs must hold M*W words and scales M*B floats")
    if server_err.numel() != plan.d or out_signs.numel() != plan.W or out_scales.numel() != plan.B:
        raise TypeError("server_err/out_signs/out_scales must hold d/W/B entries")
    rc = lib().ef_server_step(plan._h, int(M), _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                              _ptr(scales, torch.float32, "scales"),
                              _ptr(server_err, torch.float32, "server_err"), float(eta_prev), float(eta),
                              _ptr(out_signs, out_signs.dtype, "out_signs"),
                              _ptr(out_scales, torch.float32, "out_scales"), _stream_ptr(stream))
    _check(rc)


def ef_apply(plan, params, packed_signs, scales, eta, stream=None):
    if params.numel() != plan.d or packed_signs.numel() != plan.W or scales.numel() != plan.B:
        raise TypeError("params/packed_signs/scales must hold d/W/B entries")
    rc = lib().ef_apply(plan._h, _ptr(params, torch.float32, "params"),
                        _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                        _ptr(scales, torch.float32, "scales"), float(eta), _stream_ptr(stream))
    _check(rc)


def ef_apply_wd(plan, params, decay_mom, packed_signs, scales, eta, mu, lam, stream=None):
    if (params.numel() != plan.d or decay_mom.numel() != plan.d or packed_signs.numel() != plan.W
            or scales.numel() != plan.B):
        raise TypeError("params/decay_mom/packed_signs/scales must hold d/d/W/B entries")
    rc = lib().ef_apply_wd(plan._h, _ptr(params, torch.float32, "params"),
                           _ptr(decay_mom, torch.float32, "decay_mom"),
                           _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                           _ptr(scales, torch.float32, "scales"), float(eta), float(mu), float(lam),
                           _stream_ptr(stream))
    _check(rc)


def ef_payload_bytes(plan):
    return int(lib().ef_payload_bytes(plan._h))


def ef_payload_scales_offset(plan):
    return int(lib().ef_payload_scales_offset(plan._h))


def _messages(t, n, plan, name):
    """A uint8 buffer of n fused messages (Section 4.2: one message per worker)."""
    if t.numel() != n * ef_payload_bytes(plan):
        raise TypeError("%s must hold %d messages of %d bytes" % (name, n, ef_payload_bytes(plan)))
    return _ptr(t, torch.uint8, name)


def ef_worker_step_fused(plan, grad, mom, err, mu, eta_prev, eta, payloads, stream=None):
    n = 1 if grad.dim() == 1 else grad.shape[0]
    gs, ss = _stride(grad, plan.d, "grad"), _stride(mom, plan.d, "mom")
    if _stride(err, plan.d, "err") != ss or mom.shape != err.shape:
        raise TypeError("mom and err must share shape and stride")
    rc = lib().ef_worker_step_fused(plan._h, n, _ptr(grad, torch.float32, "grad"), gs,
                                    _ptr(mom, torch.float32, "mom"), _ptr(err, torch.float32, "err"), ss,
                                    float(mu), float(eta_prev), float(eta), _messages(payloads, n, plan, "payloads"),
                                    _stream_ptr(stream))
    _check(rc)


def ef_server_step_fused(plan, M, payloads, server_err, eta_prev, eta, out_payload, stream=None):
    if payloads.numel() < M * ef_payload_bytes(plan) or server_err.numel() != plan.d:
        raise TypeError("payloads must hold M messages and server_err d floats")
    rc = lib().ef_server_step_fused(plan._h, int(M), _ptr(payloads, torch.uint8, "payloads"),
                                    _ptr(server_err, torch.float32, "server_err"), float(eta_prev), float(eta),
                                    _messages(out_payload, 1, plan, "out_payload"), _stream_ptr(stream))
    _check(rc)


def ef_apply_fused(plan, params, payload, eta, stream=None):
    if params.numel() != plan.d:
        raise TypeError("params must hold d floats")
    rc = lib().ef_apply_fused(plan._h, _ptr(params, torch.float32, "params"), _messages(payload, 1, plan, "payload"),
                              float(eta), _stream_ptr(stream))
    _check(rc)


def ef_worker_step_sgd(plan, grad, err, eta_prev, eta, packed_signs, scales, stream=None):
    """Algorithm 3 worker (no momentum buffer): shapes as for ef_worker_step."""
    n = 1 if grad.dim() == 1 else grad.shape[0]
    gs, ss = _stride(grad, plan.d, "grad"), _stride(err, plan.d, "err")
    if packed_signs.numel() != n * plan.W or scales.numel() != n * plan.B:
        raise TypeError("packed_signs must hold n*W words and scales n*B floats")
    rc = lib().ef_worker_step_sgd(plan._h, n, _ptr(grad, torch.float32, "grad"), gs,
                                  _ptr(err, torch.float32, "err"), ss, float(eta_prev), float(eta),
                                  _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                                  _ptr(scales, torch.float32, "scales"), _stream_ptr(stream))
    _check(rc)


def ef_compressor_quality(plan, v, out, stream=None, static_scratch=False):
    """v: float32 [n][>=d] (or [d]); out: float64 [n][2] receives (phi, delta) per vector.
    static_scratch: go through ef_compressor_quality_static (allocates nothing, bounded size)."""
    n = 1 if v.dim() == 1 else v.shape[0]
    if out.numel() != 2 * n:
        raise TypeError("out must hold 2 doubles per vector")
    fn = lib().ef_compressor_quality_static if static_scratch else lib().ef_compressor_quality
    rc = fn(plan._h, n, _ptr(v, torch.float32, "v"), _stride(v, plan.d, "v"), _ptr(out, torch.float64, "out"),
            _stream_ptr(stream))
    _check(rc)


def ef_compressor_quality_static(plan, v, out, stream=None):
    ef_compressor_quality(plan, v, out, stream, static_scratch=True)


class State:
    """ef_state: Algorithm 4's m_i, e_i and e~ held by the library (see ef_state_create in
    include/ef.h).  Close it before its plan."""

    def __init__(self, plan, n_workers, stream=None):
        self.plan, self.n = plan, int(n_workers)
        self._h = ctypes.c_void_p()
        _check(lib().ef_state_create(plan._h, self.n, ctypes.byref(self._h), _stream_ptr(stream)))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().ef_state_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ef_state_create(plan, n_workers, stream=None):
    return State(plan, n_workers, stream)


def ef_state_destroy(state):
    state.close()


def ef_worker_step_state(plan, state, grad, mu, eta_prev, eta, packed_signs, scales, stream=None):
    n = 1 if grad.dim() == 1 else grad.shape[0]
    if n != state.n or packed_signs.numel() != n * plan.W or scales.numel() != n * plan.B:
        raise TypeError("grad must hold the state's workers; packed_signs n*W words, scales n*B floats")
    rc = lib().ef_worker_step_state(plan._h, state._h, _ptr(grad, torch.float32, "grad"), _stride(grad, plan.d, "grad"),
                                    float(mu), float(eta_prev), float(eta),
                                    _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                                    _ptr(scales, torch.float32, "scales"), _stream_ptr(stream))
    _check(rc)


def ef_server_step_state(plan, state, M, packed_signs, scales, eta_prev, eta, out_signs, out_scales, stream=None):
    if packed_signs.numel() != M * plan.W or scales.numel() != M * plan.B:
        raise TypeError("packed_signs must hold M*W words and scales M*B floats")
    if out_signs.numel() != plan.W or out_scales.numel() != plan.B:
        raise TypeError("out_signs/out_scales must hold W/B entries")
    rc = lib().ef_server_step_state(plan._h, state._h, int(M), _ptr(packed_signs, packed_signs.dtype, "packed_signs"),
                                    _ptr(scales, torch.float32, "scales"), float(eta_prev), float(eta),
                                    _ptr(out_signs, out_signs.dtype, "out_signs"),
                                    _ptr(out_scales, torch.float32, "out_scales"), _stream_ptr(stream))
    _check(rc)


def _state_copy(fn, plan, state, mom, err, server_err, stream):
    stride = plan.d
    for t, name in ((mom, "mom"), (err, "err")):
        if t is not None:
            if (1 if t.dim() == 1 else t.shape[0]) != state.n:
                raise TypeError("%s must hold the state's workers" % name)
            stride = _stride(t, plan.d, name)
    if mom is not None and err is not None and _stride(mom, plan.d, "mom") != _stride(err, plan.d, "err"):
        raise TypeError("mom and err must share their row stride")
    if server_err is not None and server_err.numel() != plan.d:
        raise TypeError("server_err must hold d entries")
    p = [None if t is None else _ptr(t, torch.float32, n) for t, n in ((mom, "mom"), (err, "err"), (server_err, "server_err"))]
    _check(fn(plan._h, state._h, p[0], p[1], stride, p[2], _stream_ptr(stream)))


def ef_state_export(plan, state, mom=None, err=None, server_err=None, stream=None):
    """Writes the true m, e ([n][>=d]) and e~ ([d]) into the given tensors (any may be None)."""
    _state_copy(lib().ef_state_export, plan, state, mom, err, server_err, stream)


def ef_state_import(plan, state, mom=None, err=None, server_err=None, stream=None):
    """Overwrites the held m, e, e~ with the given finished state (any may be None)."""
    _state_copy(lib().ef_state_import, plan, state, mom, err, server_err, stream)
