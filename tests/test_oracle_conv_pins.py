"""Pins for the convolution oracle (no GPU): short-long convolutions of CHELA Sec. 4.2, Eq. 8.

The oracle is the direct sum.  It is checked against the route the paper names for the long kernel -- Eq. 7,
y = F^-1 D_K F u, with numpy's FFT on sequences zero-padded to 2L so that the circular product of Eq. 7 equals the
causal sum -- and against closed forms, brute force and the algebra of convolution.
"""
import numpy as np
import pytest

from oracle import conv


def _rand(rng, B, d, L, m):
    return rng.standard_normal((B, d, L)), rng.standard_normal((d, m)) / m, rng.standard_normal((d, L)) / np.sqrt(L)


def test_long_conv_equals_fft_route_of_eq7():
    rng = np.random.default_rng(1)
    X, _, k = _rand(rng, 2, 3, 257, 3)
    n = 2 * 257
    want = np.fft.irfft(np.fft.rfft(X, n=n, axis=-1) * np.fft.rfft(k, n=n, axis=-1)[None], n=n, axis=-1)[..., :257]
    np.testing.assert_allclose(conv.long_conv(X, k), want, rtol=1e-10, atol=1e-11)


def test_eq7_without_padding_is_circular_and_differs():
    # as printed (DFT of size L, no padding) Eq. 7 wraps the tail of the sequence round to its start; the oracle
    # takes the zero-history reading, so it agrees with the wrapped version only where nothing has wrapped yet
    rng = np.random.default_rng(2)
    X, _, k = _rand(rng, 1, 1, 64, 3)
    k[:, 8:] = 0.0                                     # kernel of support 8
    circ = np.fft.irfft(np.fft.rfft(X, axis=-1) * np.fft.rfft(k, axis=-1)[None], n=64, axis=-1)
    got = conv.long_conv(X, k)
    np.testing.assert_allclose(got[..., 7:], circ[..., 7:], rtol=1e-10, atol=1e-11)
    assert np.abs(got[..., :7] - circ[..., :7]).max() > 1e-3


def test_long_conv_brute_force_and_special_kernels():
    rng = np.random.default_rng(3)
    X, _, k = _rand(rng, 2, 2, 9, 3)
    want = np.zeros_like(X)
    for b in range(2):
        for c in range(2):
            for t in range(9):
                for s in range(t + 1):
                    want[b, c, t] += k[c, s] * X[b, c, t - s]
    np.testing.assert_allclose(conv.long_conv(X, k), want, rtol=1e-12, atol=1e-12)
    delta = np.zeros((2, 9)); delta[:, 0] = 1.0
    np.testing.assert_array_equal(conv.long_conv(X, delta), X)                       # identity kernel
    shift = np.zeros((2, 9)); shift[:, 3] = 1.0
    np.testing.assert_array_equal(conv.long_conv(X, shift)[..., 3:], X[..., :-3])     # delay by 3
    np.testing.assert_array_equal(conv.long_conv(X, shift)[..., :3], 0 * X[..., :3])
    ones = np.ones((2, 9))
    np.testing.assert_allclose(conv.long_conv(X, ones), np.cumsum(X, axis=-1), rtol=1e-12, atol=1e-12)
    imp = np.zeros_like(X); imp[..., 0] = 1.0
    np.testing.assert_array_equal(conv.long_conv(imp, k), np.broadcast_to(k, X.shape))   # impulse response = kernel


def test_long_conv_is_causal_linear_and_commutes_with_delay():
    rng = np.random.default_rng(4)
    X, _, k = _rand(rng, 1, 2, 40, 3)
    X2 = X.copy(); X2[..., 25:] += 1.0
    assert np.array_equal(conv.long_conv(X, k)[..., :25], conv.long_conv(X2, k)[..., :25])
    a, b_ = 0.7, -1.3
    np.testing.assert_allclose(conv.long_conv(a * X + b_ * X2, k), a * conv.long_conv(X, k) + b_ * conv.long_conv(X2, k),
                               rtol=1e-12, atol=1e-12)
    Xd = np.zeros_like(X); Xd[..., 5:] = X[..., :-5]
    np.testing.assert_allclose(conv.long_conv(Xd, k)[..., 5:], conv.long_conv(X, k)[..., :-5], rtol=1e-12, atol=1e-12)


def test_short_conv_brute_force_silu_and_merge():
    rng = np.random.default_rng(5)
    X, w, _ = _rand(rng, 2, 3, 11, 4)
    lin = np.zeros_like(X)
    for t in range(11):
        for j in range(4):
            if t - j >= 0:
                lin[..., t] += w[None, :, j] * X[..., t - j]
    np.testing.assert_allclose(conv.short_conv(X, w, silu=False), lin, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(conv.short_conv(X, w, silu=True), lin / (1.0 + np.exp(-lin)), rtol=1e-12, atol=1e-12)
    # silu: known values
    one = np.ones((1, 1, 1)); w1 = np.ones((1, 1))
    assert abs(conv.short_conv(one, w1)[0, 0, 0] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-15
    assert conv.short_conv(0 * one, w1)[0, 0, 0] == 0.0
    # two parallel short kernels (size 3 and size 5) summed = one merged kernel (re-parameterisation)
    w3, w5 = rng.standard_normal((3, 3)), rng.standard_normal((3, 5))
    w3p = np.zeros((3, 5)); w3p[:, :3] = w3
    two = conv.short_conv(X, w3p, silu=False) + conv.short_conv(X, w5, silu=False)
    np.testing.assert_allclose(conv.short_conv(X, conv.merge_short_kernels(w3, w5), silu=False), two, rtol=1e-12, atol=1e-12)


def test_short_long_composition_and_channel_independence():
    rng = np.random.default_rng(6)
    X, w, k = _rand(rng, 2, 3, 30, 5)
    Z = conv.short_long_conv(X, w, k)
    np.testing.assert_array_equal(Z, conv.long_conv(conv.short_conv(X, w), k))
    for c in range(3):                                  # depthwise: channel c never sees another channel's data
        np.testing.assert_array_equal(conv.short_long_conv(X[:, c:c + 1], w[c:c + 1], k[c:c + 1]), Z[:, c:c + 1])
    np.testing.assert_array_equal(conv.short_long_conv(X, None, k), conv.long_conv(X, k))


def test_shape_errors():
    with pytest.raises(ValueError):
        conv.long_conv(np.zeros((1, 2, 8)), np.zeros((2, 7)))
    with pytest.raises(ValueError):
        conv.short_conv(np.zeros((1, 2, 8)), np.zeros((3, 3)))


# --------------------------------------------------------------------------- gradient
def test_conv_gradient_finite_differences():
    rng = np.random.default_rng(7)
    X, w, k = _rand(rng, 2, 2, 12, 4)
    dZ = rng.standard_normal(X.shape)
    dX, dw, dk = conv.short_long_conv_bwd(X, w, k, dZ)

    def loss(X_, w_, k_):
        return float((conv.short_long_conv(X_, w_, k_) * dZ).sum())

    h = 1e-6
    for which, grad in enumerate((dX, dw, dk)):
        base = [X, w, k]
        it = np.nditer(base[which], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args = [a.copy() for a in base]
            args[which][idx] += h
            up = loss(*args)
            args[which][idx] -= 2 * h
            dn = loss(*args)
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_long_conv_gradient_is_the_adjoint():
    # without the short stage Z is bilinear in (X, k): <Z, dZ> = <X, dX> = <k, dk>
    rng = np.random.default_rng(8)
    X, _, k = _rand(rng, 3, 2, 33, 3)
    dZ = rng.standard_normal(X.shape)
    dX, dw, dk = conv.short_long_conv_bwd(X, None, k, dZ)
    assert dw is None
    lhs = float((conv.long_conv(X, k) * dZ).sum())
    assert abs(lhs - float((X * dX).sum())) <= 1e-10 * max(1.0, abs(lhs))
    assert abs(lhs - float((k * dk).sum())) <= 1e-10 * max(1.0, abs(lhs))
    # the correlation with the kernel, by the library's correlate
    want = np.stack([[np.correlate(dZ[b, c], k[c], mode="full")[33 - 1:] for c in range(2)] for b in range(3)])
    np.testing.assert_allclose(dX, want, rtol=1e-11, atol=1e-12)


def test_conv_gradient_identity_kernel_reduces_to_short_stage():
    # long kernel = unit impulse: Z = silu(K_s X), so dX is the short correlation of dZ * silu'(U)
    rng = np.random.default_rng(9)
    X, w, k = _rand(rng, 1, 2, 20, 3)
    k[:] = 0.0
    k[:, 0] = 1.0
    dZ = rng.standard_normal(X.shape)
    dX, dw, dk = conv.short_long_conv_bwd(X, w, k, dZ)
    U = conv.short_conv(X, w, silu=False)
    sg = 1.0 / (1.0 + np.exp(-U))
    dU = dZ * sg * (1.0 + U * (1.0 - sg))
    want = np.zeros_like(X)
    for t in range(20):
        for j in range(3):
            if t + j < 20:
                want[..., t] += w[None, :, j] * dU[..., t + j]
    np.testing.assert_allclose(dX, want, rtol=1e-12, atol=1e-12)
