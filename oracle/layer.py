"""fp64 CPU oracle for the pieces of the CHELA layer that sit directly around the attention kernel
-- TEST INFRASTRUCTURE ONLY (same rules as the rest of this package).

Sec. 4.3, Eq. 11-12: queries and keys are not separate projections but two per-feature affine maps of ONE tensor Z,

        Q = alpha_q * Z + beta_q ,     K = alpha_k * Z + beta_k ,

with learnable alpha, beta in R^d.  With d split over H heads of width dk, each head owns its slice of the four
vectors: `affine` is a [4, H, dk] array holding (alpha_q, beta_q, alpha_k, beta_k), broadcast over batch and tokens.

Everything here is plain numpy in float64; the attention itself is the pinned C oracle.
"""
import numpy as np

from . import fwd_recurrent, bwd_recurrent


def _check(Z, affine):
    Z = np.asarray(Z, dtype=np.float64)
    affine = np.asarray(affine, dtype=np.float64)
    if Z.ndim != 4 or affine.shape != (4, Z.shape[1], Z.shape[3]):
        raise ValueError("Z must be [B,H,N,dk] and affine [4,H,dk]")
    return Z, affine


def qk_from_z(Z, affine):
    """(Q, K) of Eq. 11-12 for Z [B,H,N,dk] and affine [4,H,dk]."""
    Z, a = _check(Z, affine)
    Q = a[0][None, :, None, :] * Z + a[1][None, :, None, :]
    K = a[2][None, :, None, :] * Z + a[3][None, :, None, :]
    return Q, K


def zqk_fwd(Z, affine, V):
    """O_t = sum_{s<=t} (q_t . k_s) v_s with q, k from Eq. 11-12."""
    Q, K = qk_from_z(Z, affine)
    return fwd_recurrent(Q, K, V)


def zqk_bwd(Z, affine, V, dO):
    """(dZ, d_affine, dV) of zqk_fwd: the chain rule through Eq. 11-12.

    dZ = alpha_q * dQ + alpha_k * dK;  d_alpha_q = sum_{b,t} dQ * Z;  d_beta_q = sum_{b,t} dQ;  same for k."""
    Z, a = _check(Z, affine)
    Q, K = qk_from_z(Z, a)
    dQ, dK, dV = bwd_recurrent(Q, K, V, dO)
    dZ = a[0][None, :, None, :] * dQ + a[2][None, :, None, :] * dK
    d_aff = np.stack([(dQ * Z).sum(axis=(0, 2)), dQ.sum(axis=(0, 2)), (dK * Z).sum(axis=(0, 2)), dK.sum(axis=(0, 2))])
    return dZ, d_aff, dV


# ---------------------------------------------------------------------------------------------------------------
# Sec. 2.1 Eq. 2 as written (no mask): O = Q (K^T V), what the paper's classification models (LRA, speech, pixel
# sequences) run.  Norm is left to the caller, as in the causal case.  numpy matmul is the library step.
def noncausal_fwd(Q, K, V):
    """O[b,h] = Q[b,h] @ (K[b,h]^T @ V[b,h]): right-product linear attention without a mask."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    S = np.matmul(np.swapaxes(K, -1, -2), V)            # [B,H,dk,dv]
    return np.matmul(Q, S)


def noncausal_bwd(Q, K, V, dO):
    """(dQ, dK, dV) of noncausal_fwd: with S = K^T V and R = Q^T dO,  dQ = dO S^T, dK = V R^T, dV = K R."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    S = np.matmul(np.swapaxes(K, -1, -2), V)
    R = np.matmul(np.swapaxes(Q, -1, -2), dO)
    return np.matmul(dO, np.swapaxes(S, -1, -2)), np.matmul(V, np.swapaxes(R, -1, -2)), np.matmul(K, R)


# ---------------------------------------------------------------------------------------------------------------
# Sec. 4.3, Eq. 9: the layer's output is Norm(Q (K^T V)) * G_a, G_a a gate with the shape of the attention output.
# The paper never writes Norm out; Sec. 2.1 attributes it to the TransNormer line of work, whose attention-output
# normalisation is a root-mean-square normalisation with no learnable gain.  Reading taken here: per token and per
# head, over that head's dv features,
#
#       Norm(o) = o / sqrt(mean_j o_j^2 + eps),        Y = Norm(O) * G,
#
# eps >= 0 a small constant the caller passes (with one head this is the normalisation over the whole feature
# dimension).  The gate is an input: Eq. 10 forms it with a dense projection, which is not part of this path.
def gate_norm_fwd(O, G, eps):
    """Y = Norm(O) * G for O, G [..., dv]; Norm as defined above."""
    O, G = np.asarray(O, dtype=np.float64), np.asarray(G, dtype=np.float64)
    if O.shape != G.shape:
        raise ValueError("O and G must have the same shape")
    ms = np.mean(O * O, axis=-1, keepdims=True)
    return O / np.sqrt(ms + eps) * G


def gate_norm_bwd(O, G, dY, eps):
    """(dO, dG) of gate_norm_fwd.

    With r = (mean_j o_j^2 + eps)^(-1/2), n = r o and u = dY * G:   dG = dY * n,
    dO_j = sum_k u_k d(n_k)/d(o_j) = r (u_j - n_j mean_k(u_k n_k))   (d r / d o_j = -r^3 o_j / dv)."""
    O, G, dY = (np.asarray(x, dtype=np.float64) for x in (O, G, dY))
    if O.shape != G.shape or O.shape != dY.shape:
        raise ValueError("O, G and dY must have the same shape")
    r = 1.0 / np.sqrt(np.mean(O * O, axis=-1, keepdims=True) + eps)
    n = r * O
    u = dY * G
    dO = r * (u - n * np.mean(u * n, axis=-1, keepdims=True))
    return dO, dY * n


def gated_fwd(Q, K, V, G, eps):
    """Eq. 9 under the causal mask: (O, Y) with O the un-normalised attention output and Y = Norm(O) * G."""
    O = fwd_recurrent(Q, K, V)
    return O, gate_norm_fwd(O, G, eps)


def gated_bwd(Q, K, V, G, dY, eps):
    """(dQ, dK, dV, dG) of Y = Norm(O(Q,K,V)) * G."""
    O = fwd_recurrent(Q, K, V)
    dO, dG = gate_norm_bwd(O, G, dY, eps)
    dQ, dK, dV = bwd_recurrent(Q, K, V, dO)
    return dQ, dK, dV, dG
