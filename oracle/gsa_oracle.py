"""numpy front end of the fp64 CPU oracle (oracle/gsa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py; never by the product package.  It holds no
arithmetic of its own -- it only marshals arrays into the C functions, which
are the token-by-token recurrence of the paper's Eq. (gsa) and its
back-propagation in double precision.

Array conventions: q,k [B,T,H,dk], v [B,T,H,dv], g [B,T,H,m]; with
``cu_seqlens`` (int array [n_seqs+1]) B must be 1 and the T axis holds packed
sequences whose memories restart at every boundary.  States are
[n_seqs,H,m,d] with n_seqs = B when not packed.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def _lib():
    global _LIB
    if _LIB is None:
        # GSA_ORACLE_LIB: another build of the same source (the sanitizer run of the tests sets it)
        path = os.environ.get("GSA_ORACLE_LIB") or os.path.join(_HERE, "liboracle.so")
        if not os.path.exists(path):
            from . import build as _b  # type: ignore
            _b.build()
        lib = ctypes.CDLL(path)
        lib.gsa_oracle_num_threads.restype = ctypes.c_int
        lib.gsa_oracle_fwd.restype = ctypes.c_int
        lib.gsa_oracle_fwd.argtypes = [ctypes.c_int, _i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                       _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p,
                                       _f64p, _f64p, _f64p, _f64p]
        lib.gsa_oracle_bwd.restype = ctypes.c_int
        lib.gsa_oracle_bwd.argtypes = [ctypes.c_int, _i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                       _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p,
                                       _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p, _f64p]
        lib.gsa_oracle_decode_step.restype = ctypes.c_int
        lib.gsa_oracle_decode_step.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_double, ctypes.c_int, _f64p, _f64p, _f64p, _f64p, _f64p,
                                               _f64p, _f64p, _f64p]
        _LIB = lib
    return _LIB


def num_threads() -> int:
    return int(_lib().gsa_oracle_num_threads())


def _f64(x):
    return None if x is None else np.ascontiguousarray(x, dtype=np.float64)


def _p64(x):
    return None if x is None else x.ctypes.data_as(_f64p)


def _seqs(q, cu_seqlens):
    B, T = q.shape[0], q.shape[1]
    if cu_seqlens is None:
        cu = np.arange(B + 1, dtype=np.int32) * T
    else:
        assert B == 1, "packed sequences need B == 1"
        cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) >= 0)
    return cu


READOUTS = {"softmax": 0, "identity": 1, "swish": 2, "relu": 3, "relu2": 4}


def fwd(q, k, v, g, cu_seqlens=None, K0=None, V0=None, scale=1.0, s=None, readout="softmax"):
    """s: write intensity [B,T,H,m] (None: 1 - exp(g)).  Returns dict(o, z, KT, VT), all float64."""
    q, k, v, g, s = _f64(q), _f64(k), _f64(v), _f64(g), _f64(s)
    assert s is None or s.shape == g.shape
    B, T, H, dk = q.shape
    dv, m = v.shape[-1], g.shape[-1]
    cu = _seqs(q, cu_seqlens)
    n = len(cu) - 1
    K0, V0 = _f64(K0), _f64(V0)
    o = np.empty((B, T, H, dv), np.float64)
    z = np.empty((B, T, H, m), np.float64)
    KT = np.empty((n, H, m, dk), np.float64)
    VT = np.empty((n, H, m, dv), np.float64)
    rc = _lib().gsa_oracle_fwd(n, cu.ctypes.data_as(_i32p), H, dk, dv, m, float(scale), READOUTS[readout],
                               _p64(q), _p64(k), _p64(v), _p64(g), _p64(s), _p64(K0), _p64(V0),
                               _p64(o), _p64(z), _p64(KT), _p64(VT))
    if rc != 0:
        raise MemoryError("gsa_oracle_fwd failed")
    return dict(o=o, z=z, KT=KT, VT=VT)


def bwd(q, k, v, g, dO, cu_seqlens=None, K0=None, V0=None, dKT=None, dVT=None, scale=1.0, s=None,
        readout="softmax", intermediates=False):
    """Returns dict(dq, dk, dv, dg, dK0, dV0) and, when s is given, ds; all float64.  With
    intermediates=True also dp and dz [B,T,H,m], the gradients with respect to the read weights and the
    scores."""
    q, k, v, g, dO, s = _f64(q), _f64(k), _f64(v), _f64(g), _f64(dO), _f64(s)
    assert s is None or s.shape == g.shape
    B, T, H, dk = q.shape
    dv, m = v.shape[-1], g.shape[-1]
    cu = _seqs(q, cu_seqlens)
    n = len(cu) - 1
    K0, V0, dKT, dVT = _f64(K0), _f64(V0), _f64(dKT), _f64(dVT)
    dq = np.empty((B, T, H, dk), np.float64)
    dk_ = np.empty((B, T, H, dk), np.float64)
    dv_ = np.empty((B, T, H, dv), np.float64)
    dg = np.empty((B, T, H, m), np.float64)
    ds = None if s is None else np.empty((B, T, H, m), np.float64)
    dK0 = np.empty((n, H, m, dk), np.float64)
    dV0 = np.empty((n, H, m, dv), np.float64)
    dp = np.empty((B, T, H, m), np.float64) if intermediates else None
    dz = np.empty((B, T, H, m), np.float64) if intermediates else None
    rc = _lib().gsa_oracle_bwd(n, cu.ctypes.data_as(_i32p), H, dk, dv, m, float(scale), READOUTS[readout],
                               _p64(q), _p64(k), _p64(v), _p64(g), _p64(s), _p64(K0), _p64(V0), _p64(dO),
                               _p64(dKT), _p64(dVT),
                               _p64(dq), _p64(dk_), _p64(dv_), _p64(dg), _p64(ds), _p64(dK0), _p64(dV0), _p64(dp), _p64(dz))
    if rc != 0:
        raise MemoryError("gsa_oracle_bwd failed")
    out = dict(dq=dq, dk=dk_, dv=dv_, dg=dg, dK0=dK0, dV0=dV0)
    if ds is not None:
        out["ds"] = ds
    if intermediates:
        out["dp"], out["dz"] = dp, dz
    return out


def decode_step(q, k, v, g, K, V, scale=1.0, s=None, readout="softmax"):
    """q,k [B,H,dk], v [B,H,dv], g [B,H,m]; K [B,H,m,dk], V [B,H,m,dv] float64,
    updated IN PLACE.  Returns o [B,H,dv] float64."""
    q, k, v, g, s = _f64(q), _f64(k), _f64(v), _f64(g), _f64(s)
    assert s is None or s.shape == g.shape
    B, H, dk = q.shape
    dv, m = v.shape[-1], g.shape[-1]
    assert K.dtype == np.float64 and V.dtype == np.float64
    assert K.flags.c_contiguous and V.flags.c_contiguous
    assert K.shape == (B, H, m, dk) and V.shape == (B, H, m, dv)
    o = np.empty((B, H, dv), np.float64)
    rc = _lib().gsa_oracle_decode_step(B * H, dk, dv, m, float(scale), READOUTS[readout],
                                       _p64(q), _p64(k), _p64(v), _p64(g), _p64(s), _p64(K), _p64(V), _p64(o))
    if rc != 0:
        raise MemoryError("gsa_oracle_decode_step failed")
    return o
