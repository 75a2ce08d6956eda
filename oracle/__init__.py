"""fp64 CPU oracle for causal linear attention -- TEST INFRASTRUCTURE ONLY.

Python face of oracle/chela_oracle.c (see that file's header for the definition
and its citations: CHELA Sec. 2.1 Eq. 2, Sec. 4.1).  Inputs are numpy arrays of
shape [B, H, N, d]; they are up-cast to float64 exactly (fp32 and bf16 values
are representable) and every result is float64.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product package never does.
"""
import ctypes
import os

import numpy as np

from .build import build as _build, LIB as _LIB

_lib = None


def _load():
    global _lib
    if _lib is None:
        # CHELA_ORACLE_LIB: another build of the same source to load instead (the sanitizer build of the test tier)
        path = os.environ.get("CHELA_ORACLE_LIB") or _LIB
        if path == _LIB and (not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(
                os.path.join(os.path.dirname(_LIB), "chela_oracle.c"))):
            _build(force=True)
        _lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        for name in ("chela_oracle_fwd_quadratic", "chela_oracle_fwd_recurrent"):
            f = getattr(_lib, name)
            f.argtypes = [dp, dp, dp, dp, i, i, i, i, i]
            f.restype = None
        for name in ("chela_oracle_bwd_quadratic", "chela_oracle_bwd_recurrent"):
            f = getattr(_lib, name)
            f.argtypes = [dp, dp, dp, dp, dp, dp, dp, i, i, i, i, i]
            f.restype = None
        f = _lib.chela_oracle_fwd_state
        f.argtypes = [dp, dp, dp, dp, dp, dp, i, i, i, i, i]
        f.restype = None
        f = _lib.chela_oracle_bwd_state
        f.argtypes = [dp] * 10 + [i, i, i, i, i]
        f.restype = None
        f = _lib.chela_oracle_step
        f.argtypes = [dp, dp, dp, dp, dp, i, i, i, i]
        f.restype = None
        _lib.chela_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().chela_oracle_num_threads())


def _f64(x):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if a.ndim != 4:
        raise ValueError("expected a [B, H, N, d] array")
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(Q, K, V):
    B, H, N, dk = Q.shape
    if K.shape != Q.shape or V.shape[:3] != Q.shape[:3]:
        raise ValueError("Q, K must be [B,H,N,dk] and V [B,H,N,dv]")
    return B, H, N, dk, V.shape[3]


def _fwd(name, Q, K, V):
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H, N, dk, dv = _shapes(Q, K, V)
    O = np.empty((B, H, N, dv), dtype=np.float64)
    if O.size:
        getattr(_load(), name)(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), B, H, N, dk, dv)
    return O


def _bwd(name, Q, K, V, dO):
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    B, H, N, dk, dv = _shapes(Q, K, V)
    if dO.shape != V.shape:
        raise ValueError("dO must have V's shape")
    dQ = np.empty_like(Q)
    dK = np.empty_like(K)
    dV = np.empty_like(V)
    if Q.size and V.size:
        getattr(_load(), name)(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
                               B, H, N, dk, dv)
    else:
        dQ[...] = 0.0
        dK[...] = 0.0
        dV[...] = 0.0
    return dQ, dK, dV


def fwd_quadratic(Q, K, V):
    """O = ((Q K^T) * causal mask) V, masked parallel form (Eq. 2 + mask of Sec. 4.1)."""
    return _fwd("chela_oracle_fwd_quadratic", Q, K, V)


def fwd_recurrent(Q, K, V):
    """Token-by-token running state S += k v^T; o = S^T q (cumsum formulation, Sec. 1/3)."""
    return _fwd("chela_oracle_fwd_recurrent", Q, K, V)


def bwd_quadratic(Q, K, V, dO):
    """(dQ, dK, dV) of the quadratic form for upstream gradient dO."""
    return _bwd("chela_oracle_bwd_quadratic", Q, K, V, dO)


def bwd_recurrent(Q, K, V, dO):
    """(dQ, dK, dV) by a forward state sweep (dQ) and a reverse state sweep (dK, dV)."""
    return _bwd("chela_oracle_bwd_recurrent", Q, K, V, dO)


def _opt_state(S, B, H, dk, dv):
    if S is None:
        return None, None
    a = np.ascontiguousarray(np.asarray(S, dtype=np.float64))
    if a.shape != (B, H, dk, dv):
        raise ValueError("state must be [B, H, dk, dv]")
    return a, _ptr(a)


def fwd_state(Q, K, V, S_in=None):
    """(O, S_out) with the running state started at S_in (zero if None): segment-wise processing, Sec. 5.3."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H, N, dk, dv = _shapes(Q, K, V)
    S_in, p_in = _opt_state(S_in, B, H, dk, dv)
    O = np.empty((B, H, N, dv), dtype=np.float64)
    S_out = np.zeros((B, H, dk, dv), dtype=np.float64)
    _load().chela_oracle_fwd_state(_ptr(Q), _ptr(K), _ptr(V), p_in, _ptr(O), _ptr(S_out), B, H, N, dk, dv)
    return O, S_out


def bwd_state(Q, K, V, dO, S_in=None, dS_out=None):
    """(dQ, dK, dV, dS_in) of (Q, K, V, S_in) -> (O, S_out) for upstream gradients dO and dS_out."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    B, H, N, dk, dv = _shapes(Q, K, V)
    S_in, p_in = _opt_state(S_in, B, H, dk, dv)
    dS_out, p_out = _opt_state(dS_out, B, H, dk, dv)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(K), np.empty_like(V)
    dS_in = np.zeros((B, H, dk, dv), dtype=np.float64)
    _load().chela_oracle_bwd_state(_ptr(Q), _ptr(K), _ptr(V), p_in, _ptr(dO), p_out, _ptr(dQ), _ptr(dK), _ptr(dV),
                                   _ptr(dS_in), B, H, N, dk, dv)
    return dQ, dK, dV, dS_in


def step(q, k, v, S):
    """One decode step: returns (o, S_new) with S_new = S + k v^T and o = S_new^T q; q,k: [B,H,dk], v: [B,H,dv]."""
    q = np.ascontiguousarray(np.asarray(q, dtype=np.float64))
    k = np.ascontiguousarray(np.asarray(k, dtype=np.float64))
    v = np.ascontiguousarray(np.asarray(v, dtype=np.float64))
    S = np.array(S, dtype=np.float64, order="C", copy=True)
    B, H, dk = q.shape
    dv = v.shape[2]
    if k.shape != q.shape or v.shape[:2] != (B, H) or S.shape != (B, H, dk, dv):
        raise ValueError("shapes: q,k [B,H,dk]; v [B,H,dv]; S [B,H,dk,dv]")
    o = np.empty((B, H, dv), dtype=np.float64)
    _load().chela_oracle_step(_ptr(q), _ptr(k), _ptr(v), _ptr(S), _ptr(o), B, H, dk, dv)
    return o, S


def rel_l2(x, ref) -> float:
    """||x - ref||_2 / ||ref||_2 over the whole tensor, in float64."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((x - ref).ravel()))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
