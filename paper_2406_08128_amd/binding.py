"""Thin ctypes binding of libchela.so (see include/chela.h; measurement aids: include/chela_bench.h).

Argument marshalling only: torch tensors supply device pointers and the current HIP stream; every step of
the computation runs in the library's kernels.  There is no fallback: if the library is missing or a call
returns an error status, an exception is raised.
"""
import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchela.so")

DTYPE_BF16 = 0
DTYPE_F32 = 1

_lib = None


class ChelaError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("libchela status %d: %s" % (status, msg))
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libchela.so (built by `python -m paper_2406_08128_amd.build`); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    # CHELA_LIB: another build of the same library to load instead of the in-tree one (the sanitizer tier of the tests)
    path = os.environ.get("CHELA_LIB") or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2406_08128_amd.build` (there is no CPU fallback)" % path)
    L = ctypes.CDLL(path)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    for name in ("chela_linattn_fwd", "chela_linattn_fwd_f32", "chela_linattn_fwd_noalloc"):
        f = getattr(L, name)
        f.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
        f.restype = i
    for name in ("chela_linattn_bwd", "chela_linattn_bwd_f32"):
        f = getattr(L, name)
        f.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
        f.restype = i
    L.chela_linattn_fwd_bnhd.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_fwd_bnhd.restype = i
    L.chela_linattn_bwd_bnhd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_bwd_bnhd.restype = i
    L.chela_linattn_fwd_state.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_fwd_state.restype = i
    L.chela_linattn_bwd_state.argtypes = [vp] * 10 + [i, i, i, i, i, i, vp]
    L.chela_linattn_bwd_state.restype = i
    L.chela_linattn_zfwd.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_zfwd.restype = i
    L.chela_linattn_zbwd.argtypes = [vp] * 7 + [i, i, i, i, i, i, vp]
    L.chela_linattn_zbwd.restype = i
    L.chela_linattn_zfwd_save.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_zfwd_save.restype = i
    L.chela_linattn_zbwd_saved.argtypes = [vp] * 8 + [i, i, i, i, i, i, vp]
    L.chela_linattn_zbwd_saved.restype = i
    L.chela_linattn_z_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    L.chela_linattn_z_workspace_bytes.restype = sz
    L.chela_linattn_fwd_save.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.chela_linattn_fwd_save.restype = i
    L.chela_linattn_bwd_saved.argtypes = [vp] * 8 + [i, i, i, i, i, i, vp]
    L.chela_linattn_bwd_saved.restype = i
    L.chela_linattn_saved_bytes.argtypes = [i, i, i, i, i, i]
    L.chela_linattn_saved_bytes.restype = sz
    L.chela_linattn_train_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    L.chela_linattn_train_workspace_bytes.restype = sz
    f32 = ctypes.c_float
    L.chela_linattn_fwd_gated.argtypes = [vp] * 7 + [f32, i, i, i, i, i, i, vp]
    L.chela_linattn_fwd_gated.restype = i
    L.chela_linattn_zfwd_gated.argtypes = [vp] * 7 + [f32, i, i, i, i, i, i, vp]
    L.chela_linattn_zfwd_gated.restype = i
    L.chela_gate_norm_fwd.argtypes = [vp, vp, vp, f32, ctypes.c_longlong, i, vp]
    L.chela_gate_norm_fwd.restype = i
    L.chela_gate_norm_bwd.argtypes = [vp] * 5 + [f32, ctypes.c_longlong, i, vp]
    L.chela_gate_norm_bwd.restype = i
    L.chela_linattn_noncausal_fwd_gated.argtypes = [vp] * 6 + [f32, i, i, i, i, i, vp]
    L.chela_linattn_noncausal_fwd_gated.restype = i
    L.chela_linattn_step_gated.argtypes = [vp, vp, vp, vp, vp, vp, f32, i, i, i, i, vp]
    L.chela_linattn_step_gated.restype = i
    L.chela_linattn_noncausal_fwd.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp]
    L.chela_linattn_noncausal_fwd.restype = i
    L.chela_linattn_noncausal_bwd.argtypes = [vp] * 7 + [i, i, i, i, i, vp]
    L.chela_linattn_noncausal_bwd.restype = i
    L.chela_linattn_noncausal_workspace_bytes.argtypes = [i, i, i, i, i, i]
    L.chela_linattn_noncausal_workspace_bytes.restype = sz
    L.chela_longconv_spectrum_bytes.argtypes = [i, i]
    L.chela_longconv_spectrum_bytes.restype = sz
    L.chela_longconv_spectrum.argtypes = [vp, vp, i, i, vp]
    L.chela_longconv_spectrum.restype = i
    for name in ("chela_shortlong_conv_fwd", "chela_shortlong_conv_fwd_f32"):
        f = getattr(L, name)
        f.argtypes = [vp, vp, i, vp, vp, i, i, i, vp]
        f.restype = i
    for name in ("chela_shortlong_conv_bwd", "chela_shortlong_conv_bwd_f32"):
        f = getattr(L, name)
        f.argtypes = [vp, vp, i, vp, vp, vp, vp, vp, i, i, i, vp]
        f.restype = i
    L.chela_shortlong_conv_bwd_workspace_bytes.argtypes = [i, i, i, i, i]
    L.chela_shortlong_conv_bwd_workspace_bytes.restype = sz
    L.chela_linattn_step.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp]
    L.chela_linattn_step.restype = i
    L.chela_linattn_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    L.chela_linattn_workspace_bytes.restype = sz
    L.chela_set_workspace.argtypes = [vp, sz]
    L.chela_set_workspace.restype = i
    L.chela_get_workspace.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(sz)]
    L.chela_get_workspace.restype = i
    L.chela_status_string.argtypes = [i]
    L.chela_status_string.restype = ctypes.c_char_p
    L.chela_version.argtypes = []
    L.chela_version.restype = i
    L.chela_shutdown.argtypes = []
    L.chela_shutdown.restype = None
    L.chela_copy_probe.argtypes = [vp, vp, sz, vp]
    L.chela_copy_probe.restype = i
    L.chela_stream_probe.argtypes = [ctypes.POINTER(vp), i, ctypes.POINTER(vp), i, sz, vp]
    L.chela_stream_probe.restype = i
    L.chela_mfma_probe.argtypes = [vp, i, i, vp]
    L.chela_mfma_probe.restype = i
    L.chela_profile_enable.argtypes = [i]
    L.chela_profile_enable.restype = i
    L.chela_profile_num_kernels.argtypes = []
    L.chela_profile_num_kernels.restype = i
    L.chela_profile_kernel_name.argtypes = [i]
    L.chela_profile_kernel_name.restype = ctypes.c_char_p
    L.chela_profile_read.argtypes = [i, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ctypes.c_double)]
    L.chela_profile_read.restype = i
    L.chela_profile_reset.argtypes = []
    L.chela_profile_reset.restype = None
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().chela_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise ChelaError(status, status_string(status))


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _suffix(t: torch.Tensor) -> Tuple[str, int]:
    if t.dtype == torch.bfloat16:
        return "", DTYPE_BF16
    if t.dtype == torch.float32:
        return "_f32", DTYPE_F32
    raise TypeError("chela_linattn: tensors must be bfloat16 or float32, got %s" % t.dtype)


def _dims(Q, K, V):
    if Q.dim() != 4 or K.shape != Q.shape or V.dim() != 4 or V.shape[:3] != Q.shape[:3]:
        raise ValueError("expected Q, K: [B,H,N,dk] and V: [B,H,N,dv]")
    for t in (Q, K, V):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
        if t.dtype != Q.dtype:
            raise TypeError("all tensors must share one dtype")
    B, H, N, dk = Q.shape
    return B, H, N, dk, V.shape[3]


def chela_linattn_fwd(Q, K, V, O=None, chunk: int = 64, stream=None):
    """O = causal linear attention of (Q, K, V); enqueues on the current (or given) stream."""
    B, H, N, dk, dv = _dims(Q, K, V)
    sfx, _ = _suffix(Q)
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Q.dtype, device=Q.device)
    f = getattr(lib(), "chela_linattn_fwd" + sfx)
    with torch.cuda.device(Q.device):
        _check(f(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, dk, dv, int(chunk),
                 _stream_ptr(stream)))
    return O


def chela_linattn_fwd_noalloc(Q, K, V, O, chunk: int = 64, stream=None):
    """chela_linattn_fwd with the library's fixed scratch array: the call allocates nothing (O is the caller's)."""
    B, H, N, dk, dv = _dims(Q, K, V)
    if Q.dtype != torch.bfloat16:
        raise TypeError("chela_linattn_fwd_noalloc takes bfloat16 tensors")
    if O.shape != V.shape or O.dtype != Q.dtype or not O.is_cuda or not O.is_contiguous():
        raise ValueError("O must match V")
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_fwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, dk, dv,
                                               int(chunk), _stream_ptr(stream)))
    return O


def chela_linattn_bwd(Q, K, V, dO, dQ=None, dK=None, dV=None, chunk: int = 64, stream=None):
    """(dQ, dK, dV) for upstream gradient dO; nothing from the forward call is needed."""
    B, H, N, dk, dv = _dims(Q, K, V)
    if dO.shape != V.shape or dO.dtype != Q.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    sfx, _ = _suffix(Q)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    f = getattr(lib(), "chela_linattn_bwd" + sfx)
    with torch.cuda.device(Q.device):
        _check(f(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(),
                 dV.data_ptr(), B, H, N, dk, dv, int(chunk), _stream_ptr(stream)))
    return dQ, dK, dV


def _dims_bnhd(Q, K, V):
    if Q.dim() != 4 or K.shape != Q.shape or V.dim() != 4 or V.shape[:3] != Q.shape[:3]:
        raise ValueError("expected Q, K: [B,N,H,dk] and V: [B,N,H,dv]")
    for t in (Q, K, V):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous bf16 device tensors")
    B, N, H, dk = Q.shape
    return B, H, N, dk, V.shape[3]


def chela_linattn_fwd_bnhd(Q, K, V, O=None, stream=None):
    """O for Q, K [B,N,H,dk] and V [B,N,H,dv] (heads inside the token row); O is [B,N,H,dv]."""
    B, H, N, dk, dv = _dims_bnhd(Q, K, V)
    if O is None:
        O = torch.empty_like(V)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_fwd_bnhd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, dk, dv, 64,
                                            _stream_ptr(stream)))
    return O


def chela_linattn_bwd_bnhd(Q, K, V, dO, stream=None):
    """(dQ, dK, dV) in the [B,N,H,d] layout."""
    B, H, N, dk, dv = _dims_bnhd(Q, K, V)
    if dO.shape != V.shape or dO.dtype != V.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_bwd_bnhd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), dQ.data_ptr(),
                                            dK.data_ptr(), dV.data_ptr(), B, H, N, dk, dv, 64, _stream_ptr(stream)))
    return dQ, dK, dV


def _state_ptr(S, B, H, dk, dv, name):
    if S is None:
        return None
    if S.dtype != torch.float32 or tuple(S.shape) != (B, H, dk, dv) or not S.is_cuda or not S.is_contiguous():
        raise ValueError("%s must be a contiguous float32 device tensor [B,H,dk,dv]" % name)
    return S.data_ptr()


def chela_linattn_fwd_state(Q, K, V, S_in=None, O=None, S_out=None, chunk: int = 64, stream=None):
    """(O, S_out): forward with the running state started at S_in; S_out may be S_in (in place)."""
    B, H, N, dk, dv = _dims(Q, K, V)
    if Q.dtype != torch.bfloat16:
        raise TypeError("the stateful entry points are bf16")
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Q.dtype, device=Q.device)
    if S_out is None:
        S_out = torch.empty((B, H, dk, dv), dtype=torch.float32, device=Q.device)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_fwd_state(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                             _state_ptr(S_in, B, H, dk, dv, "S_in"), O.data_ptr(),
                                             _state_ptr(S_out, B, H, dk, dv, "S_out"), B, H, N, dk, dv, int(chunk),
                                             _stream_ptr(stream)))
    return O, S_out


def chela_linattn_bwd_state(Q, K, V, dO, S_in=None, dS_out=None, chunk: int = 64, stream=None):
    """(dQ, dK, dV, dS_in) for upstream gradients dO and dS_out."""
    B, H, N, dk, dv = _dims(Q, K, V)
    if Q.dtype != torch.bfloat16:
        raise TypeError("the stateful entry points are bf16")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dS_in = torch.empty((B, H, dk, dv), dtype=torch.float32, device=Q.device)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_bwd_state(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                             _state_ptr(S_in, B, H, dk, dv, "S_in"), dO.data_ptr(),
                                             _state_ptr(dS_out, B, H, dk, dv, "dS_out"), dQ.data_ptr(), dK.data_ptr(),
                                             dV.data_ptr(), dS_in.data_ptr(), B, H, N, dk, dv, int(chunk),
                                             _stream_ptr(stream)))
    return dQ, dK, dV, dS_in


def chela_linattn_saved_bytes(B, H, N, dk, dv, chunk=64) -> int:
    return int(lib().chela_linattn_saved_bytes(B, H, N, dk, dv, int(chunk)))


def chela_linattn_fwd_save(Q, K, V, O=None, saved=None, chunk: int = 64, stream=None):
    """(O, saved): forward that also leaves the running state at the backward's segment boundaries in `saved`."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the training pair")
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Q.dtype, device=Q.device)
    need = chela_linattn_saved_bytes(B, H, N, dk, dv, chunk)
    if saved is None:
        saved = torch.empty(max(need, 16) // 4, dtype=torch.float32, device=Q.device)
    elif saved.numel() * saved.element_size() < need or not saved.is_contiguous():
        raise ValueError("saved must be a contiguous device buffer of at least %d bytes" % need)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_fwd_save(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), saved.data_ptr(),
                                            B, H, N, dk, dv, int(chunk), _stream_ptr(stream)))
    return O, saved


def chela_linattn_bwd_saved(Q, K, V, dO, saved, dQ=None, dK=None, dV=None, chunk: int = 64, stream=None):
    """(dQ, dK, dV) using the states chela_linattn_fwd_save left for the same inputs."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the training pair")
    if dO.shape != V.shape or dO.dtype != Q.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_bwd_saved(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(),
                                             saved.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), B, H, N,
                                             dk, dv, int(chunk), _stream_ptr(stream)))
    return dQ, dK, dV


def _bf16_only(Q, what):
    if Q.dtype != torch.bfloat16:
        raise TypeError("%s is bf16 only" % what)


def chela_linattn_noncausal_fwd(Q, K, V, O=None, stream=None):
    """O = Q (K^T V) per (b,h): linear attention without a mask."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the non-causal form")
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Q.dtype, device=Q.device)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_noncausal_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, dk,
                                                 dv, _stream_ptr(stream)))
    return O


def chela_linattn_noncausal_bwd(Q, K, V, dO, stream=None):
    """(dQ, dK, dV) of chela_linattn_noncausal_fwd."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the non-causal form")
    if dO.shape != V.shape or dO.dtype != Q.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_noncausal_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(),
                                                 dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), B, H, N, dk, dv,
                                                 _stream_ptr(stream)))
    return dQ, dK, dV


def chela_linattn_noncausal_workspace_bytes(B, H, N, dk, dv, is_bwd) -> int:
    return int(lib().chela_linattn_noncausal_workspace_bytes(B, H, N, dk, dv, int(bool(is_bwd))))


def _zdims(Z, affine, V):
    if Z.dim() != 4 or V.dim() != 4 or V.shape[:3] != Z.shape[:3]:
        raise ValueError("expected Z: [B,H,N,dk] and V: [B,H,N,dv]")
    B, H, N, dk = Z.shape
    for t in (Z, V):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("Z and V must be contiguous bf16 device tensors")
    if (affine.dtype != torch.float32 or tuple(affine.shape) != (4, H, dk) or not affine.is_cuda
            or not affine.is_contiguous()):
        raise ValueError("affine must be a contiguous float32 device tensor [4,H,dk]")
    return B, H, N, dk, V.shape[3]


def chela_linattn_zfwd(Z, affine, V, O=None, chunk: int = 64, stream=None):
    """O for Q = affine[0]*Z + affine[1], K = affine[2]*Z + affine[3], formed on chip (Z is read once)."""
    B, H, N, dk, dv = _zdims(Z, affine, V)
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Z.dtype, device=Z.device)
    with torch.cuda.device(Z.device):
        _check(lib().chela_linattn_zfwd(Z.data_ptr(), affine.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, dk, dv,
                                        int(chunk), _stream_ptr(stream)))
    return O


def chela_linattn_zbwd(Z, affine, V, dO, chunk: int = 64, stream=None):
    """(dZ, d_affine, dV) of chela_linattn_zfwd for upstream gradient dO."""
    B, H, N, dk, dv = _zdims(Z, affine, V)
    if dO.shape != V.shape or dO.dtype != V.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    dZ, dV = torch.empty_like(Z), torch.empty_like(V)
    d_aff = torch.empty_like(affine)
    with torch.cuda.device(Z.device):
        _check(lib().chela_linattn_zbwd(Z.data_ptr(), affine.data_ptr(), V.data_ptr(), dO.data_ptr(), dZ.data_ptr(),
                                        d_aff.data_ptr(), dV.data_ptr(), B, H, N, dk, dv, int(chunk),
                                        _stream_ptr(stream)))
    return dZ, d_aff, dV


def chela_linattn_zfwd_save(Z, affine, V, O=None, saved=None, stream=None):
    """(O, saved): chela_linattn_zfwd that also leaves the boundary states for chela_linattn_zbwd_saved."""
    B, H, N, dk, dv = _zdims(Z, affine, V)
    if O is None:
        O = torch.empty((B, H, N, dv), dtype=Z.dtype, device=Z.device)
    need = chela_linattn_saved_bytes(B, H, N, dk, dv, 64)
    if saved is None:
        saved = torch.empty(max(need, 16) // 4, dtype=torch.float32, device=Z.device)
    elif saved.numel() * saved.element_size() < need or not saved.is_contiguous():
        raise ValueError("saved must be a contiguous device buffer of at least %d bytes" % need)
    with torch.cuda.device(Z.device):
        _check(lib().chela_linattn_zfwd_save(Z.data_ptr(), affine.data_ptr(), V.data_ptr(), O.data_ptr(),
                                             saved.data_ptr(), B, H, N, dk, dv, 64, _stream_ptr(stream)))
    return O, saved


def chela_linattn_zbwd_saved(Z, affine, V, dO, saved, stream=None):
    """(dZ, d_affine, dV) using the states chela_linattn_zfwd_save left for the same inputs."""
    B, H, N, dk, dv = _zdims(Z, affine, V)
    if dO.shape != V.shape or dO.dtype != V.dtype or not dO.is_contiguous():
        raise ValueError("dO must match V")
    dZ, dV = torch.empty_like(Z), torch.empty_like(V)
    d_aff = torch.empty_like(affine)
    with torch.cuda.device(Z.device):
        _check(lib().chela_linattn_zbwd_saved(Z.data_ptr(), affine.data_ptr(), V.data_ptr(), dO.data_ptr(),
                                              saved.data_ptr(), dZ.data_ptr(), d_aff.data_ptr(), dV.data_ptr(), B, H,
                                              N, dk, dv, 64, _stream_ptr(stream)))
    return dZ, d_aff, dV


def _gated_outputs(V, G, want_O, want_saved, dk, Y, O, saved):
    if G.shape != V.shape or G.dtype != V.dtype or not G.is_cuda or not G.is_contiguous():
        raise ValueError("G must be a contiguous device tensor shaped like V")
    for t in (Y, O):
        if t is not None and (t.shape != V.shape or t.dtype != V.dtype or not t.is_cuda or not t.is_contiguous()):
            raise ValueError("Y and O must be contiguous device tensors shaped like V")
    B, H, N, dv = V.shape
    if Y is None:
        Y = torch.empty_like(V)
    if O is None and want_O:
        O = torch.empty_like(V)
    if saved is not None or want_saved:
        need = chela_linattn_saved_bytes(B, H, N, dk, dv, 64)
        if saved is None:
            saved = torch.empty(max(need, 16) // 4, dtype=torch.float32, device=V.device)
        elif saved.numel() * saved.element_size() < need or not saved.is_contiguous():
            raise ValueError("saved must be a contiguous device buffer of at least %d bytes" % need)
    return Y, O, saved


def _ptr(t):
    return t.data_ptr() if t is not None else None


def chela_linattn_fwd_gated(Q, K, V, G, eps, want_O=False, want_saved=False, Y=None, O=None, saved=None, stream=None):
    """(Y, O, saved) with Y = Norm(O) * G (Eq. 9) formed inside the forward.  O and saved are produced when asked for
    (want_*) or when a buffer for them is passed; otherwise they come back as None."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the gated forward")
    Y, O, saved = _gated_outputs(V, G, want_O, want_saved, dk, Y, O, saved)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_fwd_gated(Q.data_ptr(), K.data_ptr(), V.data_ptr(), G.data_ptr(), _ptr(O),
                                             Y.data_ptr(), _ptr(saved), float(eps), B, H, N, dk, dv, 64,
                                             _stream_ptr(stream)))
    return Y, O, saved


def chela_linattn_zfwd_gated(Z, affine, V, G, eps, want_O=False, want_saved=False, Y=None, O=None, saved=None,
                             stream=None):
    """chela_linattn_fwd_gated with Q and K formed from Z (Eq. 11-12)."""
    B, H, N, dk, dv = _zdims(Z, affine, V)
    Y, O, saved = _gated_outputs(V, G, want_O, want_saved, dk, Y, O, saved)
    with torch.cuda.device(Z.device):
        _check(lib().chela_linattn_zfwd_gated(Z.data_ptr(), affine.data_ptr(), V.data_ptr(), G.data_ptr(), _ptr(O),
                                              Y.data_ptr(), _ptr(saved), float(eps), B, H, N, dk, dv, 64,
                                              _stream_ptr(stream)))
    return Y, O, saved


def chela_linattn_noncausal_fwd_gated(Q, K, V, G, eps, want_O=False, Y=None, O=None, stream=None):
    """(Y, O) with Y = Norm(Q (K^T V)) * G, the non-causal form with the Eq. 9 epilogue; O is None unless asked for."""
    B, H, N, dk, dv = _dims(Q, K, V)
    _bf16_only(Q, "the gated non-causal forward")
    Y, O, _ = _gated_outputs(V, G, want_O, False, dk, Y, O, None)
    with torch.cuda.device(Q.device):
        _check(lib().chela_linattn_noncausal_fwd_gated(Q.data_ptr(), K.data_ptr(), V.data_ptr(), G.data_ptr(), _ptr(O),
                                                       Y.data_ptr(), float(eps), B, H, N, dk, dv, _stream_ptr(stream)))
    return Y, O


def _gate_rows(O, G):
    if O.dim() < 1 or G.shape != O.shape:
        raise ValueError("O and G must have the same shape [..., dv]")
    for t in (O, G):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous bf16 device tensors")
    dv = O.shape[-1]
    return (O.numel() // dv if dv else 0), dv


def chela_gate_norm_fwd(O, G, eps, Y=None, stream=None):
    """Y = Norm(O) * G over the last dimension (Eq. 9 without the attention)."""
    rows, dv = _gate_rows(O, G)
    if Y is None:
        Y = torch.empty_like(O)
    elif Y.shape != O.shape or Y.dtype != O.dtype or not Y.is_cuda or not Y.is_contiguous():
        raise ValueError("Y must match O")
    with torch.cuda.device(O.device):
        _check(lib().chela_gate_norm_fwd(O.data_ptr(), G.data_ptr(), Y.data_ptr(), float(eps), rows, dv,
                                         _stream_ptr(stream)))
    return Y


def chela_gate_norm_bwd(O, G, dY, eps, in_place=False, dO=None, dG=None, stream=None):
    """(dO, dG) of chela_gate_norm_fwd; in_place=True writes dO over dY."""
    rows, dv = _gate_rows(O, G)
    if dY.shape != O.shape or dY.dtype != O.dtype or not dY.is_cuda or not dY.is_contiguous():
        raise ValueError("dY must match O")
    if in_place:
        dO = dY
    elif dO is None:
        dO = torch.empty_like(O)
    if dG is None:
        dG = torch.empty_like(O)
    for t in (dO, dG):
        if t.shape != O.shape or t.dtype != O.dtype or not t.is_cuda or not t.is_contiguous():
            raise ValueError("dO and dG must match O")
    with torch.cuda.device(O.device):
        _check(lib().chela_gate_norm_bwd(O.data_ptr(), G.data_ptr(), dY.data_ptr(), dO.data_ptr(), dG.data_ptr(),
                                         float(eps), rows, dv, _stream_ptr(stream)))
    return dO, dG


def chela_linattn_z_workspace_bytes(B, H, N, dk, dv, chunk, is_bwd) -> int:
    return int(lib().chela_linattn_z_workspace_bytes(B, H, N, dk, dv, chunk, int(bool(is_bwd))))


def chela_longconv_spectrum(k_long, stream=None):
    """Spectrum buffer of a long kernel k_long [d, L] (float32): computed once, reused for every batch."""
    if k_long.dim() != 2 or k_long.dtype != torch.float32 or not k_long.is_cuda or not k_long.is_contiguous():
        raise ValueError("k_long must be a contiguous float32 device tensor [d, L]")
    d, Lseq = k_long.shape
    nbytes = int(lib().chela_longconv_spectrum_bytes(d, Lseq))
    if nbytes == 0 and d * Lseq > 0:
        raise ValueError("sequence length %d is not supported by the long convolution" % Lseq)
    spec = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=k_long.device)
    with torch.cuda.device(k_long.device):
        _check(lib().chela_longconv_spectrum(k_long.data_ptr(), spec.data_ptr(), d, Lseq, _stream_ptr(stream)))
    return spec


def chela_shortlong_conv_fwd(X, w_short, spectrum, Z=None, stream=None):
    """Z = K_l(silu(K_s(X))) for X [B, d, L] (bf16 or float32); w_short [d, m] float32 or None; spectrum from
    chela_longconv_spectrum for the same d and L."""
    if X.dim() != 3 or not X.is_cuda or not X.is_contiguous():
        raise ValueError("X must be a contiguous device tensor [B, d, L]")
    sfx, _ = _suffix(X)
    B, d, Lseq = X.shape
    m, wp = 0, None
    if w_short is not None:
        if (w_short.dim() != 2 or w_short.shape[0] != d or w_short.dtype != torch.float32 or not w_short.is_cuda
                or not w_short.is_contiguous()):
            raise ValueError("w_short must be a contiguous float32 device tensor [d, m]")
        m, wp = w_short.shape[1], w_short.data_ptr()
    if Z is None:
        Z = torch.empty_like(X)
    f = getattr(lib(), "chela_shortlong_conv_fwd" + sfx)
    with torch.cuda.device(X.device):
        _check(f(X.data_ptr(), wp, m, spectrum.data_ptr(), Z.data_ptr(), B, d, Lseq, _stream_ptr(stream)))
    return Z


def chela_shortlong_conv_bwd(X, w_short, spectrum, dZ, stream=None):
    """(dX, d_w_short, d_k_long) of chela_shortlong_conv_fwd for the upstream gradient dZ (d_w_short is None
    without a short kernel)."""
    if X.dim() != 3 or not X.is_cuda or not X.is_contiguous() or dZ.shape != X.shape or dZ.dtype != X.dtype \
            or not dZ.is_contiguous():
        raise ValueError("X and dZ must be contiguous device tensors [B, d, L] of one dtype")
    sfx, _ = _suffix(X)
    B, d, Lseq = X.shape
    m, wp, dwp, dw = 0, None, None, None
    if w_short is not None:
        m, wp = w_short.shape[1], w_short.data_ptr()
        dw = torch.empty_like(w_short)
        dwp = dw.data_ptr()
    dX = torch.empty_like(X)
    dk = torch.empty((d, Lseq), dtype=torch.float32, device=X.device)
    f = getattr(lib(), "chela_shortlong_conv_bwd" + sfx)
    with torch.cuda.device(X.device):
        _check(f(X.data_ptr(), wp, m, spectrum.data_ptr(), dZ.data_ptr(), dX.data_ptr(), dwp, dk.data_ptr(), B, d, Lseq,
                 _stream_ptr(stream)))
    return dX, dw, dk


def chela_linattn_step(q, k, v, S, o=None, stream=None):
    """One decode step: S += k v^T in place, returns o = S^T q.  q,k: [B,H,dk] bf16, v: [B,H,dv] bf16, S fp32."""
    B, H, dk = q.shape
    dv = v.shape[2]
    if o is None:
        o = torch.empty((B, H, dv), dtype=torch.bfloat16, device=q.device)
    for t in (q, k, v, o):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("q, k, v, o must be contiguous bf16 device tensors")
    with torch.cuda.device(q.device):
        _check(lib().chela_linattn_step(q.data_ptr(), k.data_ptr(), v.data_ptr(), _state_ptr(S, B, H, dk, dv, "S"),
                                        o.data_ptr(), B, H, dk, dv, _stream_ptr(stream)))
    return o


def chela_linattn_step_gated(q, k, v, g, S, eps, y=None, stream=None):
    """One decode step with the Eq. 9 epilogue: S += k v^T in place, returns y = Norm(S^T q) * g (g: [B,H,dv] bf16)."""
    B, H, dk = q.shape
    dv = v.shape[2]
    if y is None:
        y = torch.empty((B, H, dv), dtype=torch.bfloat16, device=q.device)
    for t in (q, k, v, g, y):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("q, k, v, g, y must be contiguous bf16 device tensors")
    if g.shape != v.shape:
        raise ValueError("g must be shaped like v")
    with torch.cuda.device(q.device):
        _check(lib().chela_linattn_step_gated(q.data_ptr(), k.data_ptr(), v.data_ptr(), g.data_ptr(),
                                              _state_ptr(S, B, H, dk, dv, "S"), y.data_ptr(), float(eps), B, H, dk, dv,
                                              _stream_ptr(stream)))
    return y


def chela_linattn_workspace_bytes(B, H, N, dk, dv, chunk, is_bwd, dtype) -> int:
    return int(lib().chela_linattn_workspace_bytes(B, H, N, dk, dv, chunk, int(bool(is_bwd)), int(dtype)))


def chela_linattn_train_workspace_bytes(B, H, N, dk, dv, chunk, is_bwd) -> int:
    return int(lib().chela_linattn_train_workspace_bytes(B, H, N, dk, dv, chunk, int(bool(is_bwd))))


def chela_set_workspace(buf: Optional[torch.Tensor]) -> None:
    if buf is None:
        _check(lib().chela_set_workspace(None, 0))
    else:
        _check(lib().chela_set_workspace(buf.data_ptr(), buf.numel() * buf.element_size()))


def chela_version() -> int:
    return int(lib().chela_version())


def chela_shutdown() -> None:
    lib().chela_shutdown()


def chela_copy_probe(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """Plain streaming copy src -> dst (same byte size) by the library's copy kernel."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().chela_copy_probe(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)))


def chela_stream_probe(inputs, outputs, stream=None) -> None:
    """Plain streaming kernel that reads every tensor of `inputs` (1..4) and writes every tensor of `outputs` (1..4),
    all of one byte size: the bandwidth yardstick for a given mix of read and write streams."""
    ts = list(inputs) + list(outputs)
    nbytes = ts[0].numel() * ts[0].element_size()
    for t in ts:
        if t.numel() * t.element_size() != nbytes or not t.is_cuda or not t.is_contiguous():
            raise ValueError("all tensors must be contiguous device tensors of one byte size")
    ins = (ctypes.c_void_p * max(len(inputs), 1))(*[t.data_ptr() for t in inputs])
    outs = (ctypes.c_void_p * max(len(outputs), 1))(*[t.data_ptr() for t in outputs])
    _check(lib().chela_stream_probe(ins, len(inputs), outs, len(outputs), nbytes, _stream_ptr(stream)))


def chela_mfma_probe(out: torch.Tensor, blocks: int, iters: int, stream=None) -> int:
    """Matrix-core rate probe (registers only); `out`: at least blocks * 256 floats.  Returns the FLOP of the launch."""
    if out.dtype != torch.float32 or not out.is_cuda or out.numel() < blocks * 256:
        raise ValueError("out must be a float32 device tensor of at least blocks * 256 elements")
    _check(lib().chela_mfma_probe(out.data_ptr(), int(blocks), int(iters), _stream_ptr(stream)))
    return blocks * 4 * iters * 16 * 32768


def kernel_sources_sha256() -> str:
    """Hash of the sources the library is built from (csrc/*, in name order): what a committed profile summary was
    taken on is compared with what the tree holds now."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(_HERE, "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def chela_profile_enable(on: bool) -> None:
    _check(lib().chela_profile_enable(int(bool(on))))


def chela_profile_reset() -> None:
    lib().chela_profile_reset()


def chela_profile_read() -> dict:
    """{kernel class name: (launches, total_ms)} for the launches recorded since the last reset."""
    L = lib()
    out = {}
    for k in range(L.chela_profile_num_kernels()):
        n = ctypes.c_longlong(0)
        ms = ctypes.c_double(0.0)
        _check(L.chela_profile_read(k, ctypes.byref(n), ctypes.byref(ms)))
        if n.value:
            out[L.chela_profile_kernel_name(k).decode()] = (int(n.value), float(ms.value))
    return out
