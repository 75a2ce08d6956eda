"""The three block identities behind the convolution kernels for sequences longer than one transform, checked on the
CPU against the fp64 direct-sum oracle (numpy FFTs on small blocks stand in for the on-chip transforms):
    y_j  = sum_{i<=j} low half of circ([x_i;0], [k_{j-i}; k_{j-i-1}]),      spectrum of the operand = A_m + (-1)^bin A_{m-1}
    dv_i = sum_{j>=i} low half of the circular correlation of [dz_j;0] with the same operand,
    dk_m = low half of the inverse of D_m + (-1)^bin D_{m+1},  D_m = sum_i DZ_{i+m} conj(V_i).
A wrong sign, a swapped half or an off-by-one block index in any of them fails here, without a GPU."""
import numpy as np
import pytest

from oracle import conv as oracle_conv


def _blocks(x, bk, nb):
    out = np.zeros((nb, 2 * bk))
    for i in range(nb):
        seg = x[i * bk:(i + 1) * bk]
        out[i, :len(seg)] = seg
    return np.fft.rfft(out, axis=1)


@pytest.mark.parametrize("L,bk", [(57, 16), (64, 16), (33, 32), (100, 8)])
def test_block_identities_against_the_direct_sums(L, bk):
    rng = np.random.default_rng(L)
    nb = -(-L // bk)
    v, k, dz = (rng.standard_normal(L) for _ in range(3))
    sign = (-1.0) ** np.arange(bk + 1)
    A, V, DZ = _blocks(k, bk, nb), _blocks(v, bk, nb), _blocks(dz, bk, nb)
    G = [A[m] + (sign * A[m - 1] if m > 0 else 0.0) for m in range(nb)]
    y = np.concatenate([np.fft.irfft(sum(V[i] * G[j - i] for i in range(j + 1)))[:bk] for j in range(nb)])[:L]
    dv = np.concatenate([np.fft.irfft(sum(DZ[j] * np.conj(G[j - i]) for j in range(i, nb)))[:bk] for i in range(nb)])[:L]
    D = [sum(DZ[i + m] * np.conj(V[i]) for i in range(nb - m)) for m in range(nb)]
    dk = np.concatenate([np.fft.irfft(D[m] + (sign * D[m + 1] if m + 1 < nb else 0.0))[:bk] for m in range(nb)])[:L]
    want_y = oracle_conv.long_conv(v.reshape(1, 1, L), k.reshape(1, L))[0, 0]
    want_dv, _, want_dk = oracle_conv.short_long_conv_bwd(v.reshape(1, 1, L), None, k.reshape(1, L), dz.reshape(1, 1, L))
    assert np.abs(y - want_y).max() <= 1e-11 * (1 + np.abs(want_y).max())
    assert np.abs(dv - want_dv[0, 0]).max() <= 1e-11 * (1 + np.abs(want_dv).max())
    assert np.abs(dk - want_dk[0]).max() <= 1e-11 * (1 + np.abs(want_dk).max())
