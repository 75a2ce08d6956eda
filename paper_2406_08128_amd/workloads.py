"""Seeded synthetic inputs for causal linear attention.

This module only draws random tensors; it holds none of the method's arithmetic
and is the one piece shared by the HIP path's tests/bench and the CPU oracle's
tests.  It imports neither of them.

The five workloads are synthetic stand-ins for the shapes of the paper's
experiments (byte-level LRA Text at length 4K, Sec. 5.1; the ~200M-parameter
WikiText-103 speed benchmark of Fig. 4 / Sec. 6 Q1); the datasets themselves are
not used because the kernel's cost does not depend on the values.

Recipe: torch.Generator(cpu).manual_seed(seed); torch.randn in fp32, drawn in
the order Q, K, V, dO, each [B, H, N, d]; scaling / feature map applied in fp32;
cast to the I/O dtype (round-to-nearest-even for bf16) last.
"""
from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    dk: int
    dv: int
    dtype: str            # "f32" or "bf16": the I/O dtype
    backward: bool
    seed: int
    qk_map: str           # "gauss_over_8" or "elu1_over_128"
    chunks: tuple         # chunk sizes checked for this workload

    @property
    def token_heads(self) -> int:
        return self.B * self.H * self.N

    @property
    def tokens(self) -> int:
        return self.B * self.N


WORKLOADS: Dict[str, Workload] = {
    # Tiny fwd only, fp32 I/O.
    "tiny_f32": Workload("tiny_f32", 1, 1, 1024, 64, 64, "f32", False, 0, "gauss_over_8", (64,)),
    # LRA-shaped fwd, bf16 I/O.
    "lra_bf16": Workload("lra_bf16", 32, 8, 4096, 64, 64, "bf16", False, 1, "gauss_over_8", (64, 128)),
    # LM-shaped fwd+bwd, bf16 (d_model 768 = 12 heads x 64): the headline workload.
    "lm_bf16": Workload("lm_bf16", 4, 12, 16384, 64, 64, "bf16", True, 2, "gauss_over_8", (64,)),
    # Long-sequence fwd, bf16, positive feature map.
    "long_bf16": Workload("long_bf16", 1, 16, 65536, 128, 128, "bf16", False, 3, "elu1_over_128", (64,)),
    # Mixed-head fwd+bwd, bf16, rectangular state.
    "mixed_bf16": Workload("mixed_bf16", 8, 12, 4096, 64, 128, "bf16", True, 4, "gauss_over_8", (64,)),
}


def shrink(w: Workload, **kw) -> Workload:
    """Same recipe at a smaller (or otherwise different) shape."""
    return replace(w, **kw)


def _torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_inputs(w: Workload, with_dO: Optional[bool] = None) -> Dict[str, torch.Tensor]:
    """Return CPU tensors {"Q","K","V"[,"dO"]} in the workload's I/O dtype."""
    if with_dO is None:
        with_dO = w.backward
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    xq = torch.randn(w.B, w.H, w.N, w.dk, generator=g, dtype=torch.float32)
    xk = torch.randn(w.B, w.H, w.N, w.dk, generator=g, dtype=torch.float32)
    v = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
    if w.qk_map == "gauss_over_8":
        q, k = xq / 8.0, xk / 8.0
    elif w.qk_map == "elu1_over_128":
        q = (torch.nn.functional.elu(xq) + 1.0) / 128.0
        k = (torch.nn.functional.elu(xk) + 1.0) / 128.0
    else:
        raise ValueError(w.qk_map)
    dt = _torch_dtype(w.dtype)
    out = {"Q": q.to(dt).contiguous(), "K": k.to(dt).contiguous(), "V": v.to(dt).contiguous()}
    if with_dO:
        dO = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
        out["dO"] = dO.to(dt).contiguous()
    return out


def make_z_inputs(w: Workload, with_dO: Optional[bool] = None) -> Dict[str, torch.Tensor]:
    """Inputs for the entry points that form queries and keys from one tensor: {"Z","affine","V"[,"dO"]}.

    Recipe: generator seeded with seed + 1000; torch.randn in fp32 in the order Z [B,H,N,dk], n [4,H,dk],
    V [B,H,N,dv], dO; affine rows (scale_q, offset_q, scale_k, offset_k) = ((1 + n0/4)/8, n1/32, (1 + n2/4)/8, n3/32),
    so that queries and keys have the spread of the plain workloads (about 1/8) plus a per-feature offset;
    Z, V, dO are cast to the I/O dtype last, affine stays fp32."""
    if with_dO is None:
        with_dO = w.backward
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 1000)
    z = torch.randn(w.B, w.H, w.N, w.dk, generator=g, dtype=torch.float32)
    n = torch.randn(4, w.H, w.dk, generator=g, dtype=torch.float32)
    v = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
    affine = torch.stack([(1.0 + n[0] / 4.0) / 8.0, n[1] / 32.0, (1.0 + n[2] / 4.0) / 8.0, n[3] / 32.0]).contiguous()
    dt = _torch_dtype(w.dtype)
    out = {"Z": z.to(dt).contiguous(), "affine": affine, "V": v.to(dt).contiguous()}
    if with_dO:
        dO = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
        out["dO"] = dO.to(dt).contiguous()
    return out


def make_gate_inputs(w: Workload) -> Dict[str, torch.Tensor]:
    """Gate and output gradient for the normalised, gated output: {"G", "dY"}, both [B,H,N,dv] in the I/O dtype.

    Recipe: generator seeded with seed + 3000; torch.randn in fp32 in the order n_g, n_y; G = silu(n_g) -- the
    activation a gate leaves its projection through, so values lie in [-0.28, inf) with many near zero -- and
    dY = n_y; both cast to the I/O dtype last."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 3000)
    n_g = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
    n_y = torch.randn(w.B, w.H, w.N, w.dv, generator=g, dtype=torch.float32)
    dt = _torch_dtype(w.dtype)
    return {"G": torch.nn.functional.silu(n_g).to(dt).contiguous(), "dY": n_y.to(dt).contiguous()}


def make_conv_inputs(B: int, d: int, L: int, m: int, seed: int, dtype: str = "bf16") -> Dict[str, torch.Tensor]:
    """Inputs for the short-long convolution: {"X" [B,d,L], "w_short" [d,m], "k_long" [d,L]}.

    Recipe: generator seeded with seed + 2000; torch.randn in fp32 in the order X, n_w [d,m], n_k [d,L];
    w_short = n_w / m; k_long[c,t] = n_k[c,t] * exp(-4 t / L) * sqrt(8 / L): a decaying kernel as long as the sequence
    with unit energy, so that outputs stay of order one; X is cast to the I/O dtype last, the kernels stay fp32."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed + 2000)
    x = torch.randn(B, d, L, generator=g, dtype=torch.float32)
    nw = torch.randn(d, m, generator=g, dtype=torch.float32)
    nk = torch.randn(d, L, generator=g, dtype=torch.float32)
    t = torch.arange(L, dtype=torch.float32)
    k_long = (nk * torch.exp(-4.0 * t / L)[None, :] * (8.0 / L) ** 0.5).contiguous()
    return {"X": x.to(_torch_dtype(dtype)).contiguous(), "w_short": (nw / m).contiguous(), "k_long": k_long}


def make_growing_state_inputs(B: int, H: int, N: int, dk: int, dv: int, seed: int, device) -> Dict[str, torch.Tensor]:
    """Inputs whose running state K^T V grows linearly with the position: {"Q","K","V","dO"}, bf16, drawn ON `device`.

    Recipe: torch.Generator(device).manual_seed(seed); torch.randn in fp32 in the order x_q, x_k, x_v, x_g;
    Q = (elu(x_q) + 1) / 128, K = (elu(x_k) + 1) / 128 (the positive feature map of the long-sequence workload),
    V = silu(x_v) (what the activation in front of the values leaves: mean about 0.2, not zero), dO = x_g; cast to
    bf16 last.  Drawn on the device because the shapes this is for (hundreds of (b,h) pairs times tens of thousands
    of tokens) would take minutes and tens of GB on the host; tests copy the (b,h) pairs they hand to the oracle back."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    def draw(d):
        return torch.randn(B, H, N, d, generator=g, dtype=torch.float32, device=device)
    q = ((torch.nn.functional.elu(draw(dk)) + 1.0) / 128.0).to(torch.bfloat16)
    k = ((torch.nn.functional.elu(draw(dk)) + 1.0) / 128.0).to(torch.bfloat16)
    v = torch.nn.functional.silu(draw(dv)).to(torch.bfloat16)
    dO = draw(dv).to(torch.bfloat16)
    return {"Q": q.contiguous(), "K": k.contiguous(), "V": v.contiguous(), "dO": dO.contiguous()}


def to_f64_numpy(t: torch.Tensor):
    """Exact up-cast of an fp32/bf16 tensor to a float64 numpy array (oracle input)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
