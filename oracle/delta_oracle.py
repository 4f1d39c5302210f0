"""ctypes front end of ``delta_oracle.c`` -- TEST INFRASTRUCTURE ONLY.

The C file is the oracle of the two delta-rule rows of the paper's Table 1 (DeltaNet, Gated DeltaNet) under
Eq. 5, token by token in fp64.  This module only marshals numpy arrays (widened to float64 exactly).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "delta_oracle.c")
_LIB = os.path.join(_HERE, "libdelta_oracle.so")
_lib = None


def build_delta_oracle(force=False):
    """Compile delta_oracle.c with gcc (plain C99 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # DELTA_ORACLE_LIB: test hook of the mutation test (tests/test_oracle_meta.py), which points the pins at a
        # deliberately broken copy of the oracle to show that they notice
        path = os.environ.get("DELTA_ORACLE_LIB")
        if not path:
            build_delta_oracle()
            path = _LIB
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.delta_oracle_fwd.restype = ctypes.c_int
        lib.delta_oracle_fwd.argtypes = [ctypes.c_int] * 5 + [dp] * 9
        lib.delta_oracle_bwd.restype = ctypes.c_int
        lib.delta_oracle_bwd.argtypes = [ctypes.c_int] * 5 + [dp] * 16
        _lib = lib
    return _lib


def _f64(x, shape=None):
    if x is None:
        return None
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if shape is not None and a.shape != tuple(shape):
        raise ValueError("shape %s, expected %s" % (a.shape, tuple(shape)))
    return a


def _p(a):
    dp = ctypes.POINTER(ctypes.c_double)
    return a.ctypes.data_as(dp) if a is not None else ctypes.cast(None, dp)


def delta_oracle_fwd(q, k, v, log_alpha=None, beta=None, b=None, m0=None):
    """Return (o, m_T) in float64.  q, k: [B,H,T,dk]; v: [B,H,T,dv]; log_alpha, beta, b: [B,H,T] or None (= 1)."""
    q = _f64(q)
    B, H, T, dk = q.shape
    k = _f64(k, (B, H, T, dk))
    v = _f64(v)
    dv = v.shape[-1]
    v = _f64(v, (B, H, T, dv))
    la, be, bw = (_f64(a, (B, H, T)) for a in (log_alpha, beta, b))
    m0 = _f64(m0, (B, H, dk, dv))
    o = np.empty((B, H, T, dv), dtype=np.float64)
    mT = np.empty((B, H, dk, dv), dtype=np.float64)
    rc = _load().delta_oracle_fwd(B, H, T, dk, dv, _p(q), _p(k), _p(v), _p(la), _p(be), _p(bw), _p(m0), _p(o), _p(mT))
    if rc != 0:
        raise ValueError("delta_oracle_fwd: bad arguments")
    return o, mT


def delta_oracle_bwd(q, k, v, d_o, log_alpha=None, beta=None, b=None, m0=None, d_mT=None):
    """Return dict(dq, dk, dv, d_log_alpha, d_beta, d_b, d_m0) in float64 (None where the input was None)."""
    q = _f64(q)
    B, H, T, dk = q.shape
    k = _f64(k, (B, H, T, dk))
    v = _f64(v)
    dv = v.shape[-1]
    la, be, bw = (_f64(a, (B, H, T)) for a in (log_alpha, beta, b))
    m0 = _f64(m0, (B, H, dk, dv))
    d_o = _f64(d_o, (B, H, T, dv))
    d_mT = _f64(d_mT, (B, H, dk, dv))
    dq, dkk, dvv = np.empty((B, H, T, dk)), np.empty((B, H, T, dk)), np.empty((B, H, T, dv))
    dla, dbe, dbw = (None if a is None else np.zeros((B, H, T)) for a in (la, be, bw))
    d_m0 = np.empty((B, H, dk, dv))
    rc = _load().delta_oracle_bwd(B, H, T, dk, dv, _p(q), _p(k), _p(v), _p(la), _p(be), _p(bw), _p(m0), _p(d_o), _p(d_mT),
                                  _p(dq), _p(dkk), _p(dvv), _p(dla), _p(dbe), _p(dbw), _p(d_m0))
    if rc != 0:
        raise ValueError("delta_oracle_bwd: bad arguments")
    return dict(dq=dq, dk=dkk, dv=dvv, d_log_alpha=dla, d_beta=dbe, d_b=dbw, d_m0=d_m0)
