"""Pins for the layer-level oracle (no GPU): queries and keys as affine maps of one tensor Z (CHELA Sec. 4.3,
Eq. 11-12) around the causal linear attention.

Checked against scalar brute force, closed forms, the special case that reduces to the plain attention oracle, and
finite differences of a scalar loss -- never against a retyped copy of the oracle's own array expressions.
"""
import numpy as np
import pytest

import oracle
from oracle import layer


def _rand(rng, B, H, N, dk, dv):
    Z = rng.standard_normal((B, H, N, dk))
    aff = rng.standard_normal((4, H, dk))
    V = rng.standard_normal((B, H, N, dv))
    dO = rng.standard_normal((B, H, N, dv))
    return Z, aff, V, dO


def _brute_fwd(Z, aff, V):
    B, H, N, dk = Z.shape
    dv = V.shape[3]
    O = np.zeros((B, H, N, dv))
    for b in range(B):
        for h in range(H):
            for t in range(N):
                for s in range(t + 1):
                    dot = 0.0
                    for i in range(dk):
                        q = aff[0, h, i] * Z[b, h, t, i] + aff[1, h, i]
                        k = aff[2, h, i] * Z[b, h, s, i] + aff[3, h, i]
                        dot += q * k
                    for j in range(dv):
                        O[b, h, t, j] += dot * V[b, h, s, j]
    return O


def test_zqk_forward_brute_force():
    rng = np.random.default_rng(11)
    Z, aff, V, _ = _rand(rng, 2, 2, 6, 3, 2)
    np.testing.assert_allclose(layer.zqk_fwd(Z, aff, V), _brute_fwd(Z, aff, V), rtol=1e-12, atol=1e-12)


def test_zqk_identity_affine_is_plain_attention_of_z():
    rng = np.random.default_rng(12)
    Z, aff, V, dO = _rand(rng, 1, 3, 17, 4, 5)
    aff[0] = 1.0; aff[1] = 0.0; aff[2] = 1.0; aff[3] = 0.0
    np.testing.assert_allclose(layer.zqk_fwd(Z, aff, V), oracle.fwd_recurrent(Z, Z, V), rtol=1e-12, atol=1e-12)
    dZ, _, dV = layer.zqk_bwd(Z, aff, V, dO)
    dQ, dK, dV2 = oracle.bwd_recurrent(Z, Z, V, dO)
    np.testing.assert_allclose(dZ, dQ + dK, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dV, dV2, rtol=1e-12, atol=1e-12)


def test_zqk_offsets_only_is_scaled_cumsum():
    # alpha = 0: q and k are the constant vectors beta_q, beta_k, so O_t = (beta_q . beta_k) * sum_{s<=t} v_s
    rng = np.random.default_rng(13)
    Z, aff, V, _ = _rand(rng, 2, 2, 9, 4, 3)
    aff[0] = 0.0
    aff[2] = 0.0
    c = (aff[1] * aff[3]).sum(axis=1)                       # [H]
    want = c[None, :, None, None] * np.cumsum(V, axis=2)
    np.testing.assert_allclose(layer.zqk_fwd(Z, aff, V), want, rtol=1e-12, atol=1e-12)


def test_zqk_gradient_finite_differences():
    rng = np.random.default_rng(14)
    Z, aff, V, dO = _rand(rng, 2, 2, 5, 3, 2)
    dZ, d_aff, dV = layer.zqk_bwd(Z, aff, V, dO)

    def loss(Z_, aff_, V_):
        return float((layer.zqk_fwd(Z_, aff_, V_) * dO).sum())

    h = 1e-5
    for arr, grad, which in ((Z, dZ, 0), (aff, d_aff, 1), (V, dV, 2)):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args = [Z.copy(), aff.copy(), V.copy()]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            dn = loss(*args)
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_zqk_affine_gradient_sums_over_batch_only_within_head():
    # the parameters of head h see every batch entry of head h and nothing of the other heads
    rng = np.random.default_rng(15)
    Z, aff, V, dO = _rand(rng, 3, 2, 7, 4, 3)
    _, d_aff, _ = layer.zqk_bwd(Z, aff, V, dO)
    acc = np.zeros_like(d_aff)
    for b in range(3):
        for h in range(2):
            _, d1, _ = layer.zqk_bwd(Z[b:b + 1, h:h + 1], aff[:, h:h + 1], V[b:b + 1, h:h + 1], dO[b:b + 1, h:h + 1])
            acc[:, h] += d1[:, 0]
    np.testing.assert_allclose(d_aff, acc, rtol=1e-12, atol=1e-12)


def test_zqk_adjoint_in_v():
    # for fixed Z and affine the map V -> O is linear; dV is its adjoint applied to dO
    rng = np.random.default_rng(16)
    Z, aff, V, dO = _rand(rng, 1, 2, 12, 4, 3)
    _, _, dV = layer.zqk_bwd(Z, aff, V, dO)
    lhs = float((layer.zqk_fwd(Z, aff, V) * dO).sum())
    rhs = float((V * dV).sum())
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_zqk_shape_errors():
    with pytest.raises(ValueError):
        layer.qk_from_z(np.zeros((1, 2, 3, 4)), np.zeros((4, 1, 4)))


# --------------------------------------------------------------------------- non-causal form (Sec. 2.1, Eq. 2)
def _qkv(rng, B, H, N, dk, dv):
    return (rng.standard_normal((B, H, N, dk)), rng.standard_normal((B, H, N, dk)),
            rng.standard_normal((B, H, N, dv)), rng.standard_normal((B, H, N, dv)))


def test_noncausal_brute_force():
    rng = np.random.default_rng(21)
    Q, K, V, _ = _qkv(rng, 2, 2, 5, 3, 2)
    want = np.zeros_like(V)
    for b in range(2):
        for h in range(2):
            for t in range(5):
                for s in range(5):
                    dot = sum(Q[b, h, t, i] * K[b, h, s, i] for i in range(3))
                    for j in range(2):
                        want[b, h, t, j] += dot * V[b, h, s, j]
    np.testing.assert_allclose(layer.noncausal_fwd(Q, K, V), want, rtol=1e-12, atol=1e-12)


def test_noncausal_right_product_equals_left_product():
    # Eq. 2's point: Q (K^T V) = (Q K^T) V; the oracle takes the first, this is the second
    rng = np.random.default_rng(22)
    Q, K, V, _ = _qkv(rng, 1, 3, 40, 8, 6)
    want = np.einsum("bhts,bhsj->bhtj", np.einsum("bhti,bhsi->bhts", Q, K), V)
    np.testing.assert_allclose(layer.noncausal_fwd(Q, K, V), want, rtol=1e-11, atol=1e-11)


def test_noncausal_is_causal_plus_anticausal_minus_diagonal():
    # sum over all s = sum over s <= t  +  sum over s >= t  -  the s = t term; both one-sided sums come from the
    # pinned causal oracle (the second on the time-reversed sequence)
    rng = np.random.default_rng(23)
    Q, K, V, _ = _qkv(rng, 2, 2, 33, 4, 5)
    fwd = oracle.fwd_recurrent(Q, K, V)
    rev = oracle.fwd_recurrent(Q[:, :, ::-1], K[:, :, ::-1], V[:, :, ::-1])[:, :, ::-1]
    diag = (Q * K).sum(-1, keepdims=True) * V
    np.testing.assert_allclose(layer.noncausal_fwd(Q, K, V), fwd + rev - diag, rtol=1e-11, atol=1e-11)
    # and the last token of the causal form sees everything
    np.testing.assert_allclose(layer.noncausal_fwd(Q, K, V)[:, :, -1], fwd[:, :, -1], rtol=1e-11, atol=1e-11)


def test_noncausal_gradient_adjoint_and_finite_differences():
    rng = np.random.default_rng(24)
    Q, K, V, dO = _qkv(rng, 1, 2, 6, 3, 2)
    dQ, dK, dV = layer.noncausal_bwd(Q, K, V, dO)
    # linear in V: <O, dO> = <V, dV>; linear in Q: <O, dO> = <Q, dQ>; linear in K likewise
    lhs = float((layer.noncausal_fwd(Q, K, V) * dO).sum())
    for x, g in ((Q, dQ), (K, dK), (V, dV)):
        assert abs(lhs - float((x * g).sum())) <= 1e-10 * max(1.0, abs(lhs))
    h = 1e-5
    for which, grad in enumerate((dQ, dK, dV)):
        base = [Q, K, V]
        it = np.nditer(base[which], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args = [a.copy() for a in base]
            args[which][idx] += h
            up = float((layer.noncausal_fwd(*args) * dO).sum())
            args[which][idx] -= 2 * h
            dn = float((layer.noncausal_fwd(*args) * dO).sum())
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_noncausal_permutation_of_keys_changes_nothing():
    # without a mask the order of the (key, value) pairs is irrelevant -- the property the causal form lacks
    rng = np.random.default_rng(25)
    Q, K, V, _ = _qkv(rng, 1, 1, 20, 4, 4)
    perm = rng.permutation(20)
    np.testing.assert_allclose(layer.noncausal_fwd(Q, K[:, :, perm], V[:, :, perm]), layer.noncausal_fwd(Q, K, V),
                               rtol=1e-11, atol=1e-11)


# ------------------------------------------------------------------------------------------ Eq. 9 epilogue
# Norm(O) * G with Norm the gain-free root-mean-square normalisation over a head's features.
def test_gate_norm_hand_values():
    # one row (3, 4): mean square 12.5, so Norm = (3, 4) / sqrt(12.5); gate (2, -1)
    Y = layer.gate_norm_fwd([[3.0, 4.0]], [[2.0, -1.0]], 0.0)
    np.testing.assert_allclose(Y, [[6.0 / 12.5 ** 0.5, -4.0 / 12.5 ** 0.5]], rtol=1e-15)
    # a constant row c normalises to sign(c); eps enters under the root: row (1,1,1,1), eps = 3 -> 1/2
    np.testing.assert_allclose(layer.gate_norm_fwd([[-5.0] * 7], [[1.0] * 7], 0.0), [[-1.0] * 7], rtol=1e-15)
    np.testing.assert_allclose(layer.gate_norm_fwd([[1.0] * 4], [[1.0] * 4], 3.0), [[0.5] * 4], rtol=1e-15)


def test_gate_norm_rows_have_unit_rms_and_ignore_scale():
    rng = np.random.default_rng(5)
    O = rng.standard_normal((2, 3, 5, 8))
    ones = np.ones_like(O)
    Y = layer.gate_norm_fwd(O, ones, 0.0)
    for row in Y.reshape(-1, 8):
        assert abs(sum(x * x for x in row) / 8 - 1.0) < 1e-12
    # positive rescaling of a row changes nothing, rows do not talk to each other
    scale = rng.uniform(0.1, 10.0, size=(2, 3, 5, 1))
    np.testing.assert_allclose(layer.gate_norm_fwd(O * scale, ones, 0.0), Y, rtol=1e-12)
    O2 = O.copy()
    O2[1, 2, 3] += 1.0
    Y2 = layer.gate_norm_fwd(O2, ones, 0.0)
    changed = np.argwhere(np.abs(Y2 - Y).max(axis=-1) > 0)
    assert changed.tolist() == [[1, 2, 3]]
    # the gate multiplies feature by feature
    G = rng.standard_normal(O.shape)
    np.testing.assert_allclose(layer.gate_norm_fwd(O, G, 0.0), Y * G, rtol=1e-15)
    with pytest.raises(ValueError):
        layer.gate_norm_fwd(O, G[..., :4], 0.0)


def test_gate_norm_gradient_finite_differences_and_invariants():
    rng = np.random.default_rng(6)
    O = rng.standard_normal((2, 2, 3, 6))
    G = rng.standard_normal(O.shape)
    dY = rng.standard_normal(O.shape)
    eps = 0.05
    dO, dG = layer.gate_norm_bwd(O, G, dY, eps)

    def loss(o, g):
        return float(np.sum(layer.gate_norm_fwd(o, g, eps) * dY))

    h = 1e-6
    for idx in [(0, 0, 0, 0), (1, 1, 2, 5), (0, 1, 1, 3), (1, 0, 2, 2)]:
        E = np.zeros_like(O)
        E[idx] = h
        assert abs((loss(O + E, G) - loss(O - E, G)) / (2 * h) - dO[idx]) < 1e-8
        assert abs((loss(O, G + E) - loss(O, G - E)) / (2 * h) - dG[idx]) < 1e-8
    # without eps the map ignores the length of a row, so the gradient has no component along the row
    dO0, dG0 = layer.gate_norm_bwd(O, G, dY, 0.0)
    for o, d in zip(O.reshape(-1, 6), dO0.reshape(-1, 6)):
        assert abs(float(np.dot(o, d))) < 1e-12
    # the map is linear in the gate: <dG, G> is the loss itself
    assert abs(float(np.sum(dG * G)) - loss(O, G)) < 1e-12


def test_gated_attention_composes_and_differentiates():
    rng = np.random.default_rng(7)
    B, H, N, dk, dv = 1, 2, 5, 3, 4
    Q, K = rng.standard_normal((2, B, H, N, dk))
    V, G, dY = rng.standard_normal((3, B, H, N, dv))
    eps = 1e-3
    O, Y = layer.gated_fwd(Q, K, V, G, eps)
    np.testing.assert_allclose(O, oracle.fwd_quadratic(Q, K, V), rtol=1e-12, atol=1e-12)
    # first token: O_0 = (q_0 . k_0) v_0, so Y_0 = sign(q_0 . k_0) v_0 / sqrt(mean v_0^2 + eps / (q_0.k_0)^2) * g_0
    for h_ in range(H):
        a = float(np.dot(Q[0, h_, 0], K[0, h_, 0]))
        v = V[0, h_, 0]
        want = np.sign(a) * v / np.sqrt(np.mean(v * v) + eps / a ** 2) * G[0, h_, 0]
        np.testing.assert_allclose(Y[0, h_, 0], want, rtol=1e-12)
    dQ, dK, dV, dG = layer.gated_bwd(Q, K, V, G, dY, eps)

    def loss(q, k, v, g):
        return float(np.sum(layer.gated_fwd(q, k, v, g, eps)[1] * dY))

    h = 1e-6
    for name, X, dX in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV), ("G", G, dG)):
        for idx in [(0, 0, 0, 0), (0, 1, 4, 2), (0, 1, 2, 1)]:
            E = np.zeros_like(X)
            E[idx] = h
            args_p = [Q, K, V, G]
            args_m = [Q, K, V, G]
            pos = "QKVG".index(name)
            args_p[pos] = X + E
            args_m[pos] = X - E
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert abs(fd - dX[idx]) < 1e-7, (name, idx, fd, dX[idx])
    # causality survives the epilogue: the future does not move earlier outputs
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    Q2[:, :, 3:] += 1.0; K2[:, :, 3:] -= 2.0; V2[:, :, 3:] *= 3.0
    np.testing.assert_array_equal(layer.gated_fwd(Q2, K2, V2, G, eps)[1][:, :, :3], Y[:, :, :3])
