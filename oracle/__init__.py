"""fp64 CPU oracle of the DeltaNet layer (per-token delta rule, paper section 2.2).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the product path (the HIP library and its binding) never does, and
this package never imports the product.  The arithmetic lives in ``deltanet_oracle.c``; this
file only compiles it with gcc, loads it with ctypes and reshapes numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deltanet_oracle.c")
_LIB = os.path.join(_HERE, "libdeltanet_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle next to its source (gcc -O2 -fopenmp); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.dn_oracle_fwd.restype = ctypes.c_int
        lib.dn_oracle_fwd.argtypes = [ctypes.c_int, ip] + [ctypes.c_int] * 3 + [dp] * 7 + [ctypes.c_int]
        lib.dn_oracle_bwd.restype = ctypes.c_int
        lib.dn_oracle_bwd.argtypes = [ctypes.c_int, ip] + [ctypes.c_int] * 3 + [dp] * 12 + [ctypes.c_int]
        lib.dn_oracle_gated_fwd.restype = ctypes.c_int
        lib.dn_oracle_gated_fwd.argtypes = [ctypes.c_int, ip] + [ctypes.c_int] * 3 + [dp] * 8 + [ctypes.c_int]
        lib.dn_oracle_gated_bwd.restype = ctypes.c_int
        lib.dn_oracle_gated_bwd.argtypes = [ctypes.c_int, ip] + [ctypes.c_int] * 3 + [dp] * 14 + [ctypes.c_int]
        lib.dn_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().dn_oracle_max_threads())


def _ptr(a):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _pack(q, k, v, beta, cu_seqlens):
    """Bring [B,L,H,d] (dense) or [T,H,d] (packed, with cu_seqlens) to the packed layout."""
    q, k, v, beta = _f64(q), _f64(k), _f64(v), _f64(beta)
    if cu_seqlens is None:
        assert q.ndim == 4, "dense inputs are [B, L, H, d]"
        B, L, H, dk = q.shape
        cu = (np.arange(B + 1, dtype=np.int64) * L).astype(np.int32)
        shape = (B, L)
        q, k, v, beta = (x.reshape((B * L,) + x.shape[2:]) for x in (q, k, v, beta))
    else:
        assert q.ndim == 3, "packed inputs are [T, H, d]"
        cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
        assert cu[0] == 0 and cu[-1] == q.shape[0] and np.all(np.diff(cu) >= 0)
        shape = None
    T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (T, H, dk) and v.shape == (T, H, dv) and beta.shape == (T, H)
    return q, k, v, beta, cu, shape, (T, H, dk, dv)


def fwd(q, k, v, beta, initial_state=None, cu_seqlens=None, nthreads: int = 0):
    """(o, final_state) of the recurrence.  States are [N, H, d_k, d_v] (N = B when dense)."""
    lib = _load()
    q, k, v, beta, cu, shape, (T, H, dk, dv) = _pack(q, k, v, beta, cu_seqlens)
    N = len(cu) - 1
    S0 = _f64(initial_state)
    if S0 is not None:
        assert S0.shape == (N, H, dk, dv)
    o = np.empty((T, H, dv), dtype=np.float64)
    ST = np.empty((N, H, dk, dv), dtype=np.float64)
    rc = lib.dn_oracle_fwd(N, cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), H, dk, dv,
                           _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(S0), _ptr(o), _ptr(ST), nthreads)
    if rc != 0:
        raise RuntimeError("dn_oracle_fwd failed with %d" % rc)
    if shape is not None:
        o = o.reshape(shape + (H, dv))
    return o, ST


def bwd(q, k, v, beta, d_o, initial_state=None, dfinal_state=None, cu_seqlens=None, nthreads: int = 0):
    """(dq, dk, dv, dbeta, dinitial_state): exact gradient of sum(o*d_o) + sum(final_state*dfinal_state)."""
    lib = _load()
    q, k, v, beta, cu, shape, (T, H, dk, dv) = _pack(q, k, v, beta, cu_seqlens)
    N = len(cu) - 1
    d_o = _f64(d_o).reshape(T, H, dv)
    S0, dST = _f64(initial_state), _f64(dfinal_state)
    for s in (S0, dST):
        if s is not None:
            assert s.shape == (N, H, dk, dv)
    dq = np.empty((T, H, dk)); dkk = np.empty((T, H, dk)); dvv = np.empty((T, H, dv))
    db = np.empty((T, H)); dS0 = np.empty((N, H, dk, dv))
    rc = lib.dn_oracle_bwd(N, cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), H, dk, dv,
                           _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(S0), _ptr(d_o), _ptr(dST),
                           _ptr(dq), _ptr(dkk), _ptr(dvv), _ptr(db), _ptr(dS0), nthreads)
    if rc != 0:
        raise RuntimeError("dn_oracle_bwd failed with %d" % rc)
    if shape is not None:
        dq = dq.reshape(shape + (H, dk)); dkk = dkk.reshape(shape + (H, dk))
        dvv = dvv.reshape(shape + (H, dv)); db = db.reshape(shape + (H,))
    return dq, dkk, dvv, db, dS0


def _gate(g, shape, T, H):
    g = _f64(g)
    return g.reshape(T, H)


def gated_fwd(q, k, v, beta, g, initial_state=None, cu_seqlens=None, nthreads: int = 0):
    """(o, final_state) of the gated recurrence S_t = exp(g_t) S_{t-1} (I - beta k k^T) + beta k v^T (listing orientation)."""
    lib = _load()
    q, k, v, beta, cu, shape, (T, H, dk, dv) = _pack(q, k, v, beta, cu_seqlens)
    g = _gate(g, shape, T, H)
    N = len(cu) - 1
    S0 = _f64(initial_state)
    if S0 is not None:
        assert S0.shape == (N, H, dk, dv)
    o = np.empty((T, H, dv), dtype=np.float64)
    ST = np.empty((N, H, dk, dv), dtype=np.float64)
    rc = lib.dn_oracle_gated_fwd(N, cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), H, dk, dv,
                                 _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(g), _ptr(S0), _ptr(o), _ptr(ST), nthreads)
    if rc != 0:
        raise RuntimeError("dn_oracle_gated_fwd failed with %d" % rc)
    if shape is not None:
        o = o.reshape(shape + (H, dv))
    return o, ST


def gated_bwd(q, k, v, beta, g, d_o, initial_state=None, dfinal_state=None, cu_seqlens=None, nthreads: int = 0):
    """(dq, dk, dv, dbeta, dg, dinitial_state) of the gated recurrence."""
    lib = _load()
    q, k, v, beta, cu, shape, (T, H, dk, dv) = _pack(q, k, v, beta, cu_seqlens)
    g = _gate(g, shape, T, H)
    N = len(cu) - 1
    d_o = _f64(d_o).reshape(T, H, dv)
    S0, dST = _f64(initial_state), _f64(dfinal_state)
    for s in (S0, dST):
        if s is not None:
            assert s.shape == (N, H, dk, dv)
    dq = np.empty((T, H, dk)); dkk = np.empty((T, H, dk)); dvv = np.empty((T, H, dv))
    db = np.empty((T, H)); dg = np.empty((T, H)); dS0 = np.empty((N, H, dk, dv))
    rc = lib.dn_oracle_gated_bwd(N, cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), H, dk, dv,
                                 _ptr(q), _ptr(k), _ptr(v), _ptr(beta), _ptr(g), _ptr(S0), _ptr(d_o), _ptr(dST),
                                 _ptr(dq), _ptr(dkk), _ptr(dvv), _ptr(db), _ptr(dg), _ptr(dS0), nthreads)
    if rc != 0:
        raise RuntimeError("dn_oracle_gated_bwd failed with %d" % rc)
    if shape is not None:
        dq = dq.reshape(shape + (H, dk)); dkk = dkk.reshape(shape + (H, dk))
        dvv = dvv.reshape(shape + (H, dv)); db = db.reshape(shape + (H,)); dg = dg.reshape(shape + (H,))
    return dq, dkk, dvv, db, dg, dS0


from .prologue import feature_map, feature_map_bwd, fused_bwd, fused_fwd, sigmoid, silu  # noqa: E402,F401
