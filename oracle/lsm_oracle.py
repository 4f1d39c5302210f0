"""ctypes front end of ``lsm_oracle.c`` -- TEST INFRASTRUCTURE ONLY.

The C file is the oracle (token-by-token fp64 evaluation of paper Eq. 5 with
the Table 1 update ``k^T v`` and the read-out ``o_s = q_s M_s``).  This module
only marshals numpy arrays: every input is widened to float64 exactly (fp32
and bf16 values are representable) and handed over as contiguous buffers.
"""
import ctypes
import os
import subprocess

import numpy as np

KIND_NONE, KIND_HEAD, KIND_SCALAR, KIND_VECTOR = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsm_oracle.c")
_LIB = os.path.join(_HERE, "liblsm_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile lsm_oracle.c with gcc (plain C99 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # LSM_ORACLE_LIB: test hook of the mutation test (tests/test_oracle_meta.py), which points the pins at a
        # deliberately broken copy of the oracle to show that they notice
        path = os.environ.get("LSM_ORACLE_LIB")
        if not path:
            build_oracle()
            path = _LIB
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.lsm_oracle_fwd.restype = ctypes.c_int
        lib.lsm_oracle_fwd.argtypes = [ctypes.c_int] * 6 + [dp] * 7
        lib.lsm_oracle_bwd.restype = ctypes.c_int
        lib.lsm_oracle_bwd.argtypes = [ctypes.c_int] * 6 + [dp] * 12
        lib.lsm_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads():
    """Number of OpenMP threads the oracle will use (one per (b,h) pair at most)."""
    return int(_load().lsm_oracle_threads())


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


def _g_shape(kind, B, H, T, dk):
    return {KIND_NONE: None, KIND_HEAD: (H,), KIND_SCALAR: (B, H, T), KIND_VECTOR: (B, H, T, dk)}[kind]


def lsm_oracle_fwd(q, k, v, g, kind, m0=None):
    """Return (o, m_T) in float64.  q,k: [B,H,T,dk]; v: [B,H,T,dv]; g per kind."""
    q = _f64(q)
    B, H, T, dk = q.shape
    k = _f64(k, (B, H, T, dk))
    v = _f64(v)
    dv = v.shape[-1]
    v = _f64(v, (B, H, T, dv))
    gs = _g_shape(kind, B, H, T, dk)
    g = _f64(g, gs) if gs is not None else None
    m0 = _f64(m0, (B, H, dk, dv))
    o = np.empty((B, H, T, dv), dtype=np.float64)
    mT = np.empty((B, H, dk, dv), dtype=np.float64)
    rc = _load().lsm_oracle_fwd(B, H, T, dk, dv, kind, _p(q), _p(k), _p(v), _p(g), _p(m0), _p(o), _p(mT))
    if rc != 0:
        raise ValueError("lsm_oracle_fwd: bad arguments")
    return o, mT


def lsm_oracle_bwd(q, k, v, g, kind, d_o, m0=None, d_mT=None):
    """Return dict(dq, dk, dv, dg, d_m0) in float64; dg is None for kind none."""
    q = _f64(q)
    B, H, T, dk = q.shape
    k = _f64(k, (B, H, T, dk))
    v = _f64(v)
    dv = v.shape[-1]
    gs = _g_shape(kind, B, H, T, dk)
    g = _f64(g, gs) if gs is not None else None
    m0 = _f64(m0, (B, H, dk, dv))
    d_o = _f64(d_o, (B, H, T, dv))
    d_mT = _f64(d_mT, (B, H, dk, dv))
    dq = np.empty((B, H, T, dk))
    dkk = np.empty((B, H, T, dk))
    dvv = np.empty((B, H, T, dv))
    dg = np.zeros(gs) if gs is not None else None
    d_m0 = np.empty((B, H, dk, dv))
    rc = _load().lsm_oracle_bwd(B, H, T, dk, dv, kind, _p(q), _p(k), _p(v), _p(g), _p(m0),
                                _p(d_o), _p(d_mT), _p(dq), _p(dkk), _p(dvv), _p(dg), _p(d_m0))
    if rc != 0:
        raise ValueError("lsm_oracle_bwd: bad arguments")
    return dict(dq=dq, dk=dkk, dv=dvv, dg=dg, d_m0=d_m0)
