"""ctypes binding of the C oracle (la2_oracle.c); compiles it with gcc when needed.

TEST INFRASTRUCTURE ONLY.  All arrays are numpy float64, C-contiguous,
[batch, heads, n, d]; lambda is float64 [heads].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "la2_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)


def build(force=False):
    """Compile la2_oracle.c -> liboracle.so (gcc, OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # LA2_ORACLE_LIB: a build of la2_oracle.c made elsewhere (the sanitizer test's instrumented one)
        path = os.environ.get("LA2_ORACLE_LIB")
        if not path:
            build()
            path = _LIB
        _lib = ctypes.CDLL(path)
        _lib.la2_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().la2_oracle_num_threads())


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return a.ctypes.data_as(_dp)


def _shape4(q):
    if q.ndim != 4:
        raise ValueError("expected [batch, heads, n, d]")
    return q.shape


def _lam(lam, H):
    lam = np.ascontiguousarray(np.broadcast_to(np.asarray(lam, dtype=np.float64), (H,)))
    return lam


def fwd_direct(q, k, v, lam):
    q, k, v = _f64(q), _f64(k), _f64(v)
    b, H, n, d = _shape4(q)
    lam = _lam(lam, H)
    o = np.empty_like(q)
    _load().la2_oracle_fwd_direct(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int64(n), ctypes.c_int(d), _p(q), _p(k), _p(v), _p(lam), _p(o)
    )
    return o


def bwd_direct(q, k, v, d_o, lam):
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    b, H, n, d = _shape4(q)
    lam = _lam(lam, H)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    _load().la2_oracle_bwd_direct(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int64(n), ctypes.c_int(d),
        _p(q), _p(k), _p(v), _p(d_o), _p(lam), _p(dq), _p(dk), _p(dv),
    )
    return dq, dk, dv


def fwd_recurrent(q, k, v, lam, kv_init=None, return_state=False):
    q, k, v = _f64(q), _f64(k), _f64(v)
    b, H, n, d = _shape4(q)
    lam = _lam(lam, H)
    o = np.empty_like(q)
    kvf = np.empty((b, H, d, d), dtype=np.float64)
    init = None
    if kv_init is not None:
        init = _f64(kv_init)
        assert init.shape == (b, H, d, d)
    _load().la2_oracle_fwd_recurrent(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int64(n), ctypes.c_int(d),
        _p(q), _p(k), _p(v), _p(lam), _p(init) if init is not None else None, _p(o), _p(kvf),
    )
    return (o, kvf) if return_state else o


def bwd_recurrent(q, k, v, d_o, lam):
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    b, H, n, d = _shape4(q)
    lam = _lam(lam, H)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    _load().la2_oracle_bwd_recurrent(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int64(n), ctypes.c_int(d),
        _p(q), _p(k), _p(v), _p(d_o), _p(lam), _p(dq), _p(dk), _p(dv),
    )
    return dq, dk, dv


def bwd_recurrent_state(q, k, v, d_o, lam, kv_init=None, d_kv_final=None):
    """Backward of one segment: gradients of a loss that depends on the segment's outputs (d_o) and
    on its final state (d_kv_final), for a segment that started from kv_init.
    Returns dq, dk, dv, d_kv_init."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    b, H, n, d = _shape4(q)
    lam = _lam(lam, H)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    dkv0 = np.empty((b, H, d, d), dtype=np.float64)
    init = _f64(kv_init) if kv_init is not None else None
    dfin = _f64(d_kv_final) if d_kv_final is not None else None
    for a in (init, dfin):
        assert a is None or a.shape == (b, H, d, d)
    _load().la2_oracle_bwd_recurrent_state(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int64(n), ctypes.c_int(d),
        _p(q), _p(k), _p(v), _p(d_o), _p(lam),
        _p(init) if init is not None else None, _p(dfin) if dfin is not None else None,
        _p(dq), _p(dk), _p(dv), _p(dkv0),
    )
    return dq, dk, dv, dkv0


def decode_step(q, k, v, lam, kv):
    """One recurrent step.  q, k, v: [b, H, d]; kv: [b, H, d, d] float64, updated in place.
    Returns o [b, H, d] computed from the UPDATED state."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    b, H, d = q.shape
    lam = _lam(lam, H)
    if kv.dtype != np.float64 or not kv.flags["C_CONTIGUOUS"] or kv.shape != (b, H, d, d):
        raise ValueError("kv must be C-contiguous float64 [b, H, d, d]")
    o = np.empty_like(q)
    _load().la2_oracle_decode_step(
        ctypes.c_int(b), ctypes.c_int(H), ctypes.c_int(d), _p(q), _p(k), _p(v), _p(lam), _p(kv), _p(o)
    )
    return o


def fwd_rows(q, k, v, lam, rows):
    """Direct form for selected positions of ONE head.  q, k, v: [n, d]; lam: scalar."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    n, d = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    out = np.empty((rows.size, d), dtype=np.float64)
    _load().la2_oracle_fwd_rows(
        ctypes.c_int64(n), ctypes.c_int(d), _p(q), _p(k), _p(v), ctypes.c_double(float(lam)),
        ctypes.c_int64(rows.size), rows.ctypes.data_as(_ip), _p(out),
    )
    return out


def bwd_rows(q, k, v, d_o, lam, rows):
    """Direct-form gradients for selected positions of ONE head.  Returns dq, dk, dv rows."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    n, d = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    dq = np.empty((rows.size, d), dtype=np.float64)
    dk = np.empty_like(dq)
    dv = np.empty_like(dq)
    _load().la2_oracle_bwd_rows(
        ctypes.c_int64(n), ctypes.c_int(d), _p(q), _p(k), _p(v), _p(d_o), ctypes.c_double(float(lam)),
        ctypes.c_int64(rows.size), rows.ctypes.data_as(_ip), _p(dq), _p(dk), _p(dv),
    )
    return dq, dk, dv
