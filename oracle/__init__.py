"""ctypes front end of the CPU oracle (oracle/ef_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

Every wrapper takes and returns numpy arrays; state arrays (m, e, te, x) are
updated in place exactly as Algorithm 4 of the paper updates them.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ef_oracle.c")
_LIB = os.path.join(_HERE, "libef_oracle.so")
# tests/test_pins_catch_mistakes.py points this at a copy of the source with a planted mistake
# to show that the pins notice it; nothing else sets it.
if os.environ.get("EF_ORACLE_SRC"):
    _SRC = os.path.abspath(os.environ["EF_ORACLE_SRC"])
    _LIB = os.path.splitext(_SRC)[0] + ".so"

# -ffp-contract=off: every fp32 operation of Algorithm 4 rounds once, no FMA.
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-shared",
          "-fPIC", "-Wall", "-Wextra"]


def build(force=False):
    """Compile ef_oracle.c with gcc (single-threaded plain C)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc"] + CFLAGS + ["-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_i64p = ctypes.POINTER(ctypes.c_int64)


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.efo_sign_words.restype = ctypes.c_int64
        L.efo_sign_words.argtypes = [ctypes.c_int64]
        L.efo_check_offsets.argtypes = [_i64p, ctypes.c_int64, ctypes.c_int64]
        L.efo_compress.argtypes = [_f32p, ctypes.c_int64, _i64p, ctypes.c_int64, _u64p, _f32p]
        L.efo_decode.argtypes = [_u64p, _f32p, ctypes.c_int64, _i64p, ctypes.c_int64, _f32p]
        L.efo_worker_step.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int64, _i64p, ctypes.c_int64,
                                      ctypes.c_float, ctypes.c_float, ctypes.c_float, _u64p, _f32p]
        L.efo_worker_step_sgd.argtypes = [_f32p, _f32p, ctypes.c_int64, _i64p, ctypes.c_int64,
                                          ctypes.c_float, ctypes.c_float, _u64p, _f32p]
        L.efo_server_step.argtypes = [ctypes.c_int, _u64p, _f32p, _f32p, ctypes.c_int64, _i64p,
                                      ctypes.c_int64, ctypes.c_float, ctypes.c_float, _u64p, _f32p]
        L.efo_apply.argtypes = [_f32p, _u64p, _f32p, ctypes.c_int64, _i64p, ctypes.c_int64,
                                ctypes.c_float]
        L.efo_apply_wd.argtypes = [_f32p, _f32p, _u64p, _f32p, ctypes.c_int64, _i64p, ctypes.c_int64,
                                   ctypes.c_float, ctypes.c_float, ctypes.c_float]
        L.efo_quality.argtypes = [_f32p, ctypes.c_int64, _i64p, ctypes.c_int64,
                                  ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.efo_step.argtypes = [ctypes.c_int, _f32p, _f32p, _f32p, _f32p, _f32p, ctypes.c_int64,
                               _i64p, ctypes.c_int64, ctypes.c_float, ctypes.c_float,
                               ctypes.c_float, _u64p, _f32p, _u64p, _f32p]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def _chk(rc, what):
    if rc != 0:
        raise OracleError("%s failed with oracle code %d" % (what, rc))


def _arr(a, dtype, name, writable=False):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous numpy array of %s" % (name, np.dtype(dtype)))
    if writable and not a.flags["WRITEABLE"]:
        raise TypeError("%s must be writable" % name)
    return a


def _f(a):
    return a.ctypes.data_as(_f32p)


def _u(a):
    return a.ctypes.data_as(_u64p)


def _i(a):
    return a.ctypes.data_as(_i64p)


def sign_words(d):
    return int(lib().efo_sign_words(int(d)))


def _offs(offsets):
    offs = np.ascontiguousarray(offsets, dtype=np.int64)
    if offs.ndim != 1 or offs.size < 2:
        raise OracleError("block_offsets must hold B+1 >= 2 entries")
    return offs, offs.size - 1


def compress(v, offsets):
    """C_B(v) -> (signs uint64[W], scales float32[B])."""
    v = _arr(v, np.float32, "v")
    offs, B = _offs(offsets)
    d = v.size
    signs = np.zeros(sign_words(d), dtype=np.uint64)
    scales = np.zeros(B, dtype=np.float32)
    _chk(lib().efo_compress(_f(v), d, _i(offs), B, _u(signs), _f(scales)), "efo_compress")
    return signs, scales


def decode(signs, scales, offsets):
    """Payload -> the vector Delta it stands for (float32[d])."""
    signs = _arr(signs, np.uint64, "signs")
    scales = _arr(scales, np.float32, "scales")
    offs, B = _offs(offsets)
    d = int(offs[-1])
    if signs.size != sign_words(d) or scales.size != B:
        raise OracleError("payload size does not match block_offsets")
    out = np.empty(d, dtype=np.float32)
    _chk(lib().efo_decode(_u(signs), _f(scales), d, _i(offs), B, _f(out)), "efo_decode")
    return out


def worker_step(g, m, e, offsets, mu, eta_prev, eta):
    """One worker, one iteration.  m and e are updated in place."""
    g = _arr(g, np.float32, "g")
    m = _arr(m, np.float32, "m", True)
    e = _arr(e, np.float32, "e", True)
    offs, B = _offs(offsets)
    d = g.size
    if m.size != d or e.size != d:
        raise OracleError("g, m, e must have equal length")
    signs = np.zeros(sign_words(d), dtype=np.uint64)
    scales = np.zeros(B, dtype=np.float32)
    _chk(lib().efo_worker_step(_f(g), _f(m), _f(e), d, _i(offs), B, mu, eta_prev, eta,
                               _u(signs), _f(scales)), "efo_worker_step")
    return signs, scales


def worker_step_sgd(g, e, offsets, eta_prev, eta):
    """One worker of Algorithm 3 (no momentum), one iteration.  e is updated in place."""
    g = _arr(g, np.float32, "g")
    e = _arr(e, np.float32, "e", True)
    offs, B = _offs(offsets)
    d = g.size
    if e.size != d:
        raise OracleError("g, e must have equal length")
    signs = np.zeros(sign_words(d), dtype=np.uint64)
    scales = np.zeros(B, dtype=np.float32)
    _chk(lib().efo_worker_step_sgd(_f(g), _f(e), d, _i(offs), B, eta_prev, eta, _u(signs), _f(scales)),
         "efo_worker_step_sgd")
    return signs, scales


def server_step(signs, scales, te, offsets, eta_prev, eta):
    """signs uint64[M][W], scales float32[M][B]; te updated in place."""
    signs = _arr(signs, np.uint64, "signs")
    scales = _arr(scales, np.float32, "scales")
    te = _arr(te, np.float32, "te", True)
    offs, B = _offs(offsets)
    d = te.size
    W = sign_words(d)
    if signs.ndim != 2 or scales.ndim != 2 or signs.shape[0] != scales.shape[0]:
        raise OracleError("signs and scales must be [M][W] and [M][B]")
    M = signs.shape[0]
    if signs.shape[1] != W or scales.shape[1] != B:
        raise OracleError("payload size does not match block_offsets")
    out_signs = np.zeros(W, dtype=np.uint64)
    out_scales = np.zeros(B, dtype=np.float32)
    _chk(lib().efo_server_step(M, _u(signs), _f(scales), _f(te), d, _i(offs), B, eta_prev, eta,
                               _u(out_signs), _f(out_scales)), "efo_server_step")
    return out_signs, out_scales


def apply(x, signs, scales, offsets, eta):
    """x <- x - eta * decode(signs, scales), in place."""
    x = _arr(x, np.float32, "x", True)
    signs = _arr(signs, np.uint64, "signs")
    scales = _arr(scales, np.float32, "scales")
    offs, B = _offs(offsets)
    d = x.size
    if signs.size != sign_words(d) or scales.size != B:
        raise OracleError("payload size does not match block_offsets")
    _chk(lib().efo_apply(_f(x), _u(signs), _f(scales), d, _i(offs), B, eta), "efo_apply")


def apply_wd(x, mt, signs, scales, offsets, eta, mu, lam):
    """Appendix A update with weight decay: mt <- mu*mt + lam*x; x <- x - eta*(decode + mu*mt + lam*x)."""
    x = _arr(x, np.float32, "x", True)
    mt = _arr(mt, np.float32, "mt", True)
    signs = _arr(signs, np.uint64, "signs")
    scales = _arr(scales, np.float32, "scales")
    offs, B = _offs(offsets)
    d = x.size
    if mt.size != d or signs.size != sign_words(d) or scales.size != B:
        raise OracleError("sizes do not match block_offsets")
    _chk(lib().efo_apply_wd(_f(x), _f(mt), _u(signs), _f(scales), d, _i(offs), B, eta, mu, lam), "efo_apply_wd")


def quality(v, offsets):
    """(phi(v) of Proposition 1, delta(v) of the non-block compressor of Eq. (1))."""
    v = _arr(v, np.float32, "v")
    offs, B = _offs(offsets)
    phi, delta = ctypes.c_double(), ctypes.c_double()
    _chk(lib().efo_quality(_f(v), v.size, _i(offs), B, ctypes.byref(phi), ctypes.byref(delta)), "efo_quality")
    return phi.value, delta.value


def step(g, m, e, te, x, offsets, mu, eta_prev, eta):
    """One whole iteration: g, m, e are float32[M][d]; m, e, te, x updated in
    place.  Returns (wsigns [M][W], wscales [M][B], ssigns [W], sscales [B])."""
    g = _arr(g, np.float32, "g")
    m = _arr(m, np.float32, "m", True)
    e = _arr(e, np.float32, "e", True)
    te = _arr(te, np.float32, "te", True)
    x = _arr(x, np.float32, "x", True)
    offs, B = _offs(offsets)
    if g.ndim != 2 or m.shape != g.shape or e.shape != g.shape:
        raise OracleError("g, m, e must be [M][d]")
    M, d = g.shape
    if te.size != d or x.size != d:
        raise OracleError("te and x must have length d")
    W = sign_words(d)
    wsigns = np.zeros((M, W), dtype=np.uint64)
    wscales = np.zeros((M, B), dtype=np.float32)
    ssigns = np.zeros(W, dtype=np.uint64)
    sscales = np.zeros(B, dtype=np.float32)
    _chk(lib().efo_step(M, _f(g), _f(m), _f(e), _f(te), _f(x), d, _i(offs), B, mu, eta_prev, eta,
                        _u(wsigns), _f(wscales), _u(ssigns), _f(sscales)), "efo_step")
    return wsigns, wscales, ssigns, sscales
