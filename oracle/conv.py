"""fp64 CPU oracle for the short-long convolutions (CHELA Sec. 4.2, Eq. 8) -- TEST INFRASTRUCTURE ONLY.

Python face of the two convolution routines in oracle/chela_oracle.c (direct sums, O(L^2) for the long kernel).
Tensors are [B, d, L] (time fastest); w_short is [d, m] (the merged short kernel), k_long is [d, L].
"""
import ctypes

import numpy as np

from . import _load


def _c(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def merge_short_kernels(w3, wm):
    """The two parallel short kernels (size 3 and size m >= 3) as one size-m kernel: taps are added lag by lag
    (structural re-parameterisation, Sec. 4.2)."""
    w3, wm = _c(w3), _c(wm)
    out = wm.copy()
    out[:, :3] += w3
    return out


def short_conv(X, w_short, silu=True):
    X, w = _c(X), _c(w_short)
    B, d, L = X.shape
    if w.ndim != 2 or w.shape[0] != d:
        raise ValueError("w_short must be [d, m]")
    V = np.empty_like(X)
    lib = _load()
    lib.chela_oracle_short_conv.restype = None
    lib.chela_oracle_short_conv(_p(X), _p(w), _p(V), ctypes.c_int(B), ctypes.c_int(d), ctypes.c_int(L),
                                ctypes.c_int(w.shape[1]), ctypes.c_int(1 if silu else 0))
    return V


def long_conv(V, k_long):
    V, k = _c(V), _c(k_long)
    B, d, L = V.shape
    if k.shape != (d, L):
        raise ValueError("k_long must be [d, L]")
    Y = np.empty_like(V)
    lib = _load()
    lib.chela_oracle_long_conv.restype = None
    lib.chela_oracle_long_conv(_p(V), _p(k), _p(Y), ctypes.c_int(B), ctypes.c_int(d), ctypes.c_int(L))
    return Y


def short_long_conv(X, w_short, k_long):
    """Z = K_l(silu(K_s(X))) (Eq. 8); w_short None skips the short stage and the activation (plain long convolution)."""
    V = _c(X) if w_short is None else short_conv(X, w_short, silu=True)
    return long_conv(V, k_long)


def short_long_conv_bwd(X, w_short, k_long, dZ):
    """(dX, dw_short, dk_long) of short_long_conv for the upstream gradient dZ; dw_short is None if w_short is."""
    X, k, dZ = _c(X), _c(k_long), _c(dZ)
    B, d, L = X.shape
    if k.shape != (d, L) or dZ.shape != X.shape:
        raise ValueError("shapes: X, dZ [B,d,L]; k_long [d,L]")
    dX, dk = np.empty_like(X), np.empty_like(k)
    lib = _load()
    lib.chela_oracle_short_long_conv_bwd.restype = None
    if w_short is None:
        lib.chela_oracle_short_long_conv_bwd(_p(X), None, ctypes.c_int(0), _p(k), _p(dZ), _p(dX), None, _p(dk),
                                             ctypes.c_int(B), ctypes.c_int(d), ctypes.c_int(L))
        return dX, None, dk
    w = _c(w_short)
    dw = np.empty_like(w)
    lib.chela_oracle_short_long_conv_bwd(_p(X), _p(w), ctypes.c_int(w.shape[1]), _p(k), _p(dZ), _p(dX), _p(dw), _p(dk),
                                         ctypes.c_int(B), ctypes.c_int(d), ctypes.c_int(L))
    return dX, dw, dk
