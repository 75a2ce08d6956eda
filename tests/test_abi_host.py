"""Host-side checks of the C ABI (no GPU): the library loads, exports every declared symbol, and rejects bad
arguments before any HIP call."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("chela.h", "chela_bench.h")]


@pytest.fixture(scope="module")
def L():
    from paper_2406_08128_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2406_08128_amd.build import build
        build(verbose=False)
    return binding.lib()


def _declared_symbols():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(chela_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared_symbols()
    assert "chela_linattn_fwd" in names and "chela_linattn_bwd" in names and len(names) >= 9
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings(L):
    assert L.chela_version() == 100
    for code in range(0, -9, -1):
        s = L.chela_status_string(code).decode()
        assert s.startswith("CHELA_")
    assert b"unknown" in L.chela_status_string(-99)


A = 0x10000        # fake, aligned, non-null "device pointers": validation must reject before touching them
SZ = 1 << 30


def _fwd(L, name="chela_linattn_fwd", Q=A, K=A + SZ, V=A + 2 * SZ, O=A + 3 * SZ, B=1, H=1, N=64, dk=64, dv=64,
         chunk=64):
    return getattr(L, name)(Q, K, V, O, B, H, N, dk, dv, chunk, None)


def _bwd(L, name="chela_linattn_bwd", Q=A, K=A + SZ, V=A + 2 * SZ, dO=A + 3 * SZ, dQ=A + 4 * SZ, dK=A + 5 * SZ,
         dV=A + 6 * SZ, B=1, H=1, N=64, dk=64, dv=64, chunk=64):
    return getattr(L, name)(Q, K, V, dO, dQ, dK, dV, B, H, N, dk, dv, chunk, None)


@pytest.mark.parametrize("name", ["chela_linattn_fwd", "chela_linattn_fwd_f32", "chela_linattn_fwd_bnhd",
                                  "chela_linattn_fwd_noalloc"])
def test_fwd_argument_errors(L, name):
    assert _fwd(L, name, Q=None) == -1
    assert _fwd(L, name, O=None) == -1
    assert _fwd(L, name, B=-1) == -2
    assert _fwd(L, name, N=-5) == -2
    assert _fwd(L, name, dk=48) == -3
    assert _fwd(L, name, dv=256) == -3
    assert _fwd(L, name, chunk=7) == -4
    assert _fwd(L, name, chunk=0) == -4
    assert _fwd(L, name, K=A + SZ + 2) == -5
    assert _fwd(L, name, O=A + 8) == -5
    assert _fwd(L, name, O=A) == -6                       # output == Q
    assert _fwd(L, name, O=A + 2 * SZ + 64) == -6         # output overlaps V
    # empty problems succeed without touching anything, even with null pointers
    assert _fwd(L, name, N=0, Q=None, K=None, V=None, O=None) == 0
    assert _fwd(L, name, B=0) == 0
    assert _fwd(L, name, H=0) == 0


def test_noalloc_forward_rejects_states_beyond_its_fixed_array(L):
    # decided on the host from the plan, before any HIP call: 149 sequences of two million tokens with 128 x 128 states
    B, H, N, dk, dv = 1, 149, 1984972, 128, 128
    assert L.chela_linattn_workspace_bytes(B, H, N, dk, dv, 64, 0, 0) > (32 << 20)
    big = 1 << 40
    assert L.chela_linattn_fwd_noalloc(A, A + big, A + 2 * big, A + 3 * big, B, H, N, dk, dv, 64, None) == -7


def test_chunk_sets_differ_by_dtype(L):
    assert _fwd(L, "chela_linattn_fwd", chunk=32) == -4
    assert _fwd(L, "chela_linattn_fwd_f32", chunk=128) == -4


@pytest.mark.parametrize("name", ["chela_linattn_bwd", "chela_linattn_bwd_f32", "chela_linattn_bwd_bnhd"])
def test_bwd_argument_errors(L, name):
    assert _bwd(L, name, dO=None) == -1
    assert _bwd(L, name, dV=None) == -1
    assert _bwd(L, name, H=-2) == -2
    assert _bwd(L, name, dk=32) == -3
    assert _bwd(L, name, chunk=1) == -4
    assert _bwd(L, name, dK=A + 5 * SZ + 4) == -5
    assert _bwd(L, name, dQ=A + 3 * SZ) == -6             # dQ == dO
    assert _bwd(L, name, dK=A + 4 * SZ) == -6             # dK == dQ
    assert _bwd(L, name, N=0) == 0


def test_state_and_step_argument_errors(L):
    f = L.chela_linattn_fwd_state
    S = A + 8 * SZ
    assert f(A, A + SZ, A + 2 * SZ, S + 4, A + 3 * SZ, None, 1, 1, 64, 64, 64, 64, None) == -5   # misaligned state
    assert f(A, A + SZ, A + 2 * SZ, A + 3 * SZ, A + 3 * SZ, None, 1, 1, 64, 64, 64, 64, None) == -6   # O overlaps S_in
    assert f(None, A + SZ, A + 2 * SZ, None, A + 3 * SZ, None, 1, 1, 64, 64, 64, 64, None) == -1
    g = L.chela_linattn_bwd_state
    assert g(A, A + SZ, A + 2 * SZ, None, A + 3 * SZ, None, A + 4 * SZ, A + 5 * SZ, A + 6 * SZ, A + 4 * SZ,
             1, 1, 64, 64, 64, 64, None) == -6                                                     # dS_in overlaps dQ
    assert g(A, A + SZ, A + 2 * SZ, None, A + 3 * SZ, None, A + 4 * SZ, A + 5 * SZ, A + 6 * SZ, None,
             1, 1, 64, 48, 64, 64, None) == -3
    st = L.chela_linattn_step
    assert st(A, A + SZ, A + 2 * SZ, S, A + 3 * SZ, 0, 4, 64, 64, None) == 0
    assert st(A, A + SZ, A + 2 * SZ, None, A + 3 * SZ, 1, 4, 64, 64, None) == -1
    assert st(A, A + SZ, A + 2 * SZ, S, A + 3 * SZ, 1, 4, 64, 96, None) == -3
    assert st(A, A + SZ, A + 2 * SZ, S, S, 1, 4, 64, 64, None) == -6
    assert st(A, A + SZ, A + 2 * SZ, S + 4, A + 3 * SZ, 1, 4, 64, 64, None) == -5
    assert st(A, A + SZ, A + 2 * SZ, S, A + 3 * SZ, -1, 4, 64, 64, None) == -2


def test_z_entry_point_argument_errors(L):
    f, g, w = L.chela_linattn_zfwd, L.chela_linattn_zbwd, L.chela_linattn_z_workspace_bytes
    Z, AF, V, O = A, A + SZ, A + 2 * SZ, A + 3 * SZ
    assert f(None, AF, V, O, 1, 2, 64, 64, 64, 64, None) == -1
    assert f(Z, None, V, O, 1, 2, 64, 64, 64, 64, None) == -1
    assert f(Z, AF + 4, V, O, 1, 2, 64, 64, 64, 64, None) == -5
    assert f(Z, AF, V, AF, 1, 2, 64, 64, 64, 64, None) == -6          # O on top of the parameters
    assert f(Z, AF, V, O, 1, 2, 64, 96, 64, 64, None) == -3
    assert f(Z, AF, V, O, 1, 2, 64, 64, 64, 32, None) == -4
    assert f(None, None, None, None, 1, 2, 0, 64, 64, 64, None) == 0
    dZ, dA, dV, dO = A + 4 * SZ, A + 5 * SZ, A + 6 * SZ, A + 7 * SZ
    assert g(Z, AF, V, dO, dZ, None, dV, 1, 2, 64, 64, 64, 64, None) == -1
    assert g(Z, AF, V, dO, dZ, AF, dV, 1, 2, 64, 64, 64, 64, None) == -6   # d_affine on top of affine
    assert g(Z, AF, V, dO, dZ, dA, dZ, 1, 2, 64, 64, 64, 64, None) == -6   # dV on top of dZ
    assert g(Z, AF, V, dO, dZ, dA, dV, -1, 2, 64, 64, 64, 64, None) == -2
    assert w(1, 2, 0, 64, 64, 64, 0) == 0 and w(1, 2, 64, 64, 48, 64, 0) == 0
    # one segment, forward: nothing; backward: the workgroups' shares of the parameter gradients, [B*H][4][dk] fp32
    assert w(1, 2, 64, 64, 64, 64, 0) == 0
    assert w(1, 2, 64, 64, 64, 64, 1) == 2 * 4 * 64 * 4
    SV = A + 9 * SZ
    fs, gs = L.chela_linattn_zfwd_save, L.chela_linattn_zbwd_saved
    assert fs(Z, AF, V, O, None, 1, 2, 64, 64, 64, 64, None) == -1
    assert fs(Z, AF, V, O, SV + 8, 1, 2, 64, 64, 64, 64, None) == -5
    assert fs(Z, AF, V, O, V, 1, 2, 64, 64, 64, 64, None) == -6
    assert gs(Z, AF, V, dO, None, dZ, dA, dV, 1, 2, 64, 64, 64, 64, None) == -1
    assert gs(Z, AF, V, dO, SV, dZ, SV, dV, 1, 2, 64, 64, 64, 64, None) == -6
    big = w(4, 12, 16384, 64, 64, 64, 1)
    plain = L.chela_linattn_workspace_bytes(4, 12, 16384, 64, 64, 64, 1, 0)
    assert big > plain and (big - plain) % (48 * 4 * 64 * 4) == 0


def test_training_pair_argument_errors(L):
    f, g, sb = L.chela_linattn_fwd_save, L.chela_linattn_bwd_saved, L.chela_linattn_saved_bytes
    Q, K, V, O, SV = A, A + SZ, A + 2 * SZ, A + 3 * SZ, A + 8 * SZ
    assert sb(1, 1, 64, 64, 64, 64) == 64 * 64 * 4              # one segment: the state at the end of the sequence
    assert sb(0, 1, 64, 64, 64, 64) == 0 and sb(1, 1, 64, 64, 96, 64) == 0 and sb(1, 1, 64, 64, 64, 32) == 0
    big = sb(4, 12, 16384, 64, 64, 64)
    assert big > 0 and big % (48 * 64 * 64 * 4) == 0 and big // (48 * 64 * 64 * 4) <= 64
    assert f(Q, K, V, O, None, 1, 1, 64, 64, 64, 64, None) == -1
    assert f(Q, K, V, O, SV + 4, 1, 1, 64, 64, 64, 64, None) == -5
    assert f(Q, K, V, O, O, 1, 1, 64, 64, 64, 64, None) == -6
    assert f(Q, K, V, O, SV, 1, 1, 64, 64, 64, 16, None) == -4
    assert f(None, None, None, None, None, 1, 1, 0, 64, 64, 64, None) == 0
    dO, dQ, dK, dV = A + 3 * SZ, A + 4 * SZ, A + 5 * SZ, A + 6 * SZ
    assert g(Q, K, V, dO, None, dQ, dK, dV, 1, 1, 64, 64, 64, 64, None) == -1
    assert g(Q, K, V, dO, SV, dQ, SV, dV, 1, 1, 64, 64, 64, 64, None) == -6      # dK on top of the saved states
    assert g(Q, K, V, dO, SV, dQ, dK, dV, 1, 1, 64, 128, 256, 64, None) == -3


def test_noncausal_argument_errors(L):
    f, g, w = L.chela_linattn_noncausal_fwd, L.chela_linattn_noncausal_bwd, L.chela_linattn_noncausal_workspace_bytes
    Q, K, V, O = A, A + SZ, A + 2 * SZ, A + 3 * SZ
    assert f(None, K, V, O, 1, 1, 64, 64, 64, None) == -1
    assert f(Q, K, V, None, 1, 1, 64, 64, 64, None) == -1
    assert f(Q, K, V, O + 2, 1, 1, 64, 64, 64, None) == -5
    assert f(Q, K, V, K, 1, 1, 64, 64, 64, None) == -6
    assert f(Q, K, V, O, 1, 1, 64, 64, 80, None) == -3
    assert f(Q, K, V, O, 1, -1, 64, 64, 64, None) == -2
    assert f(None, None, None, None, 1, 1, 0, 64, 64, None) == 0
    dO, dQ, dK, dV = A + 3 * SZ, A + 4 * SZ, A + 5 * SZ, A + 6 * SZ
    assert g(Q, K, V, None, dQ, dK, dV, 1, 1, 64, 64, 64, None) == -1
    assert g(Q, K, V, dO, dQ, dQ, dV, 1, 1, 64, 64, 64, None) == -6
    assert g(Q, K, V, dO, dQ, dK, dV, 0, 1, 64, 64, 64, None) == 0
    assert w(1, 1, 64, 64, 64, 0) == 64 * 64 * 4 and w(1, 1, 64, 64, 64, 1) == 2 * 64 * 64 * 4
    assert w(1, 1, 0, 64, 64, 0) == 0 and w(1, 1, 64, 64, 72, 0) == 0
    # the scratch is bounded by the GPU's size, not by N
    assert w(4, 12, 1 << 20, 64, 64, 0) <= 600 * 64 * 64 * 4


def test_conv_argument_errors(L):
    sb, sp, f = L.chela_longconv_spectrum_bytes, L.chela_longconv_spectrum, L.chela_shortlong_conv_fwd
    # the (K[k], K[M-k]) pairs; for 4096 < L <= 16384 also the copy the matrix-core kernel reads (32768 complex
    # half-precision numbers and a scale per channel), each of the two parts rounded up to 256 bytes
    up = lambda n: (n + 255) // 256 * 256
    assert sb(3, 4096) == 3 * 2049 * 16 and sb(0, 64) == 0
    # beyond 16384 steps: one spectrum per channel and block of 16384 steps, up to 2^20 steps
    assert sb(3, 16385) == 3 * 2 * 8193 * 16 and sb(2, 65536) == 2 * 4 * 8193 * 16 and sb(1, 65537) == 5 * 8193 * 16
    assert sb(1, 1 << 20) == 64 * 8193 * 16 and sb(3, (1 << 20) + 1) == 0
    assert sb(3, 16384) == up(3 * 8193 * 16) + 3 * 32768 * 4 + up(3 * 4)
    assert sb(2, 257) == 2 * 513 * 16 and sb(2, 256) == 2 * 129 * 16 and sb(1, 1) == 129 * 16
    K, S, X, W, Y = A, A + SZ, A + 2 * SZ, A + 3 * SZ, A + 4 * SZ
    assert sp(None, S, 4, 100, None) == -1
    assert sp(K, S + 8, 4, 100, None) == -5
    assert sp(K, S, 4, (1 << 20) + 1, None) == -2
    assert sp(K, K, 4, 100, None) == -6
    assert sp(K, S, 0, 100, None) == 0
    assert f(None, W, 9, S, Y, 2, 4, 100, None) == -1
    assert f(X, W, 0, S, Y, 2, 4, 100, None) == -2
    assert f(X, W, 33, S, Y, 2, 4, 100, None) == -2
    assert f(X, W, 9, S, Y, 2, 4, (1 << 20) + 1, None) == -2
    assert f(X, W, 9, S, X, 2, 4, 100, None) == -6
    assert f(X, W, 9, S, Y + 6, 2, 4, 100, None) == -5
    assert f(X, None, 0, S, Y, 0, 4, 100, None) == 0


def test_conv_bwd_argument_errors(L):
    g, wsb = L.chela_shortlong_conv_bwd, L.chela_shortlong_conv_bwd_workspace_bytes
    X, W, S, dZ, dX, dW, dK = A, A + SZ, A + 2 * SZ, A + 3 * SZ, A + 4 * SZ, A + 5 * SZ, A + 6 * SZ
    # one sequence: a single workgroup per channel, no shares of the long-kernel gradient to keep
    assert wsb(1, 4, 100, 1, 0) == 1 * 4 * (100 * 4 + 128) and wsb(1, 4, 100, 1, 1) == 1 * 4 * (100 * 4 + 128)
    assert wsb(1, 4, 100, 0, 0) == 0 and wsb(2, 4, 100, 1, 7) == 0
    # few channels: the sequences are dealt out to G workgroups per channel (G = 2 here, at most the batch size), each
    # leaving d * (M/2 + 1) pairs of sums
    assert wsb(2, 4, 100, 0, 0) == 2 * 4 * 129 * 16
    assert wsb(2, 4, 100, 1, 0) == 2 * 4 * 129 * 16 + 2 * 4 * (100 * 4 + 128)
    # enough channels to fill the GPU: one workgroup per channel again
    assert wsb(8, 16384, 100, 0, 0) == 0
    # at the largest transform size the running sums live in the workspace whatever G is
    assert wsb(1, 4, 16001, 0, 0) == 4 * 8193 * 16 and wsb(1, 4, 16000, 0, 1) == 4 * 8193 * 16
    # bf16 I/O with 4096 < L <= 16384, L a multiple of 8: room for the matrix-core kernel as well (a spectrum of
    # half-precision pairs for each of 256 workgroups), whichever of the two kernels runs
    assert wsb(1, 4, 16000, 0, 0) == 256 * 32768 * 4
    assert wsb(2, 4, 16000, 0, 1) == 2 * 4 * 8193 * 16
    assert wsb(2, 4, 16000, 1, 1) == 2 * 4 * 8193 * 16 + 2 * 4 * (16000 * 4 + 8 * 128)
    assert wsb(2, 4, 16000, 1, 0) == 256 * 32768 * 4 + 2 * 4 * (16000 * 4 + 8 * 128)
    # beyond 16384 steps: one running sum per channel and block distance, whatever the batch size and I/O type
    assert wsb(3, 4, 40000, 0, 0) == 4 * 3 * 8193 * 16 and wsb(1, 4, 40000, 0, 1) == 4 * 3 * 8193 * 16
    assert wsb(2, 4, 40000, 1, 0) == 4 * 3 * 8193 * 16 + 2 * 4 * (40000 * 4 + 20 * 128)
    assert g(None, W, 9, S, dZ, dX, dW, dK, 2, 4, 100, None) == -1
    assert g(X, W, 9, S, dZ, dX, None, dK, 2, 4, 100, None) == -1
    assert g(X, W, 33, S, dZ, dX, dW, dK, 2, 4, 100, None) == -2          # at most 32 taps, as in the forward
    assert g(X, W, 9, S, dZ, dX, dW, dK, 2, 4, (1 << 20) + 1, None) == -2
    assert g(X, W, 9, S, dZ, X, dW, dK, 2, 4, 100, None) == -6
    assert g(X, W, 9, S, dZ, dX, dW, dX, 2, 4, 100, None) == -6
    assert g(X, W, 9, S, dZ + 2, dX, dW, dK, 2, 4, 100, None) == -5
    assert g(X, W, 9, S, dZ, dX, dW, dK, 2, 0, 100, None) == 0


def test_shape_overflow_is_rejected(L):
    assert _fwd(L, B=1 << 20, H=1 << 20, N=1 << 20) == -2


def test_workspace_bytes(L):
    w = L.chela_linattn_workspace_bytes
    assert w(0, 1, 64, 64, 64, 64, 0, 0) == 0
    assert w(1, 1, 64, 64, 64, 64, 0, 0) == 64 * 64 * 4           # one segment: one slot, used only with a carried-in state
    assert w(1, 1, 64, 48, 64, 64, 0, 0) == 0                     # invalid -> 0
    state = 48 * 64 * 64 * 4                                      # one fp32 state for each of the 48 (b,h) pairs
    fwd = w(4, 12, 16384, 64, 64, 64, 0, 0)
    bwd = w(4, 12, 16384, 64, 64, 64, 1, 0)
    assert fwd > 0 and fwd % state == 0                           # forward: one state array (K^T V prefixes)
    assert bwd > 0 and bwd % (2 * state) == 0                     # backward: two (prefix of V^T K, suffix of dO^T Q)
    assert 2 <= fwd // state <= 64 and 2 <= bwd // (2 * state) <= 64
    # 256 or more (b,h) pairs need no segmentation: one slot per pair, touched only when a state is carried in
    assert w(32, 8, 4096, 64, 64, 64, 0, 0) == 256 * 64 * 64 * 4
    # fixed-memory property: the number of segments is set by the GPU, not by N, so the scratch stays bounded
    for n in (1 << 16, 1 << 18, 1 << 20):
        assert w(4, 12, n, 64, 64, 64, 0, 0) <= 64 * state
        # (the bf16 backward keeps its segments within 8192 tokens: two states per 8192 tokens and pair, no more)
        assert 2 * (n // 8192) * state <= w(4, 12, n, 64, 64, 64, 1, 0) <= 2 * max(64, n // 8192) * state


def test_planner_stays_within_its_bounds_over_random_shapes(L):
    # whatever the shape, the split is between one segment and one segment per chunk, small problems included, and
    # the scratch stays a whole number of states per (b,h) pair
    import random
    rnd = random.Random(20240611)
    w = L.chela_linattn_workspace_bytes
    for _ in range(3000):
        B, H = rnd.randint(1, 40), rnd.randint(1, 40)
        N = rnd.choice([1, 63, 64, 65, 200, 1000, 1024, 4096, 5000, 16384, 100000, 1 << 20])
        dk, dv = rnd.choice([64, 128]), rnd.choice([64, 128])
        for dtype, chunks in ((0, (64, 128)), (1, (16, 32, 64))):
            for bwd in (0, 1):
                chunk = rnd.choice(chunks)
                ws = w(B, H, N, dk, dv, chunk, bwd, dtype)
                # (the query covers every call of its kind -- with and without carried states, the training pair --
                # so it is a whole number of states per pair, at most two arrays of them)
                per_state = B * H * dk * dv * 4
                arrays = 2 if (bwd and dtype == 0) else 1
                assert ws % per_state == 0, (B, H, N, dk, dv, chunk, bwd, dtype, ws)
                n_seg = max(1, ws // (per_state * arrays))         # (no scratch at all: a single segment)
                smallest_chunk = 32 if dtype == 1 else 64          # what the kernels tile with at the least
                assert 1 <= n_seg <= (N + smallest_chunk - 1) // smallest_chunk
                assert n_seg <= 32768                              # segments ride on a secondary grid dimension
                if B * H > 256 and (N <= 8192 or dtype == 1):
                    assert n_seg == 1                              # (longer bf16 sequences: the backward's walk is capped;
                                                                   #  exactly 256: the bf16 backward may cut each in two)
                if dtype == 0 and not bwd:
                    # the forward of the training pair cuts at least where its backward will keep a state
                    tw = L.chela_linattn_train_workspace_bytes(B, H, N, dk, dv, chunk, 0)
                    sv = L.chela_linattn_saved_bytes(B, H, N, dk, dv, chunk)
                    assert tw % per_state == 0 and (tw >= sv or sv == per_state)


def test_forward_query_covers_the_training_pairs_forward(L):
    # 96 (b,h) pairs of 65536 tokens: the plain forward plans 5 segments, the forward that saves states for the backward
    # cuts where the backward will (whose walk is capped at 8192 tokens), 10 times per sequence: a query of its own
    state = 64 * 64 * 4
    assert L.chela_linattn_train_workspace_bytes(8, 12, 65536, 64, 64, 64, 0) >= 96 * 10 * state
    assert L.chela_linattn_workspace_bytes(8, 12, 65536, 64, 64, 64, 0, 0) < 96 * 10 * state


def test_backward_walk_is_capped(L):
    # bf16 backward: no segment is longer than 8192 tokens unless the sweep checkpoints its own first pass
    # (a single segment without carried states): 300 pairs of 65536 tokens need 7 copies each, or, with carried
    # states, two arrays of 8 segments
    state = 64 * 64 * 4
    assert L.chela_linattn_workspace_bytes(300, 1, 65536, 64, 64, 64, 1, 0) == 300 * 2 * 8 * state


def test_the_method_header_declares_no_measurement_aid():
    text = re.sub(r"/\*.*?\*/", "", open(HEADERS[0]).read(), flags=re.S)
    assert "chela_copy_probe" not in text and "chela_stream_probe" not in text and "chela_profile_" not in text
    bench = re.sub(r"/\*.*?\*/", "", open(HEADERS[1]).read(), flags=re.S)
    assert "chela_linattn" not in bench


def test_caller_scratch_is_per_host_thread(L):
    # every thread sets a buffer of its own (fake, aligned addresses: nothing is ever dereferenced) and must keep
    # seeing it while the others set and reset theirs
    import threading
    L.chela_get_workspace.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_size_t)]
    L.chela_get_workspace.restype = ctypes.c_int
    L.chela_set_workspace.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    errors = []
    barrier = threading.Barrier(8)

    def worker(k):
        mine, size = 0x100000 * (k + 1), 4096 * (k + 1)
        p, n = ctypes.c_void_p(), ctypes.c_size_t()
        barrier.wait()
        for it in range(2000):
            if L.chela_set_workspace(mine, size) != 0:
                errors.append((k, "set"))
            L.chela_get_workspace(ctypes.byref(p), ctypes.byref(n))
            if p.value != mine or n.value != size:
                errors.append((k, it, p.value, n.value))
            # a problem that needs more scratch than this thread's buffer holds is refused on this thread's account
            if _fwd(L, B=4, H=12, N=16384) != -7:
                errors.append((k, it, "not refused"))
            if it % 3 == k % 3:
                L.chela_set_workspace(None, 0)
                L.chela_get_workspace(ctypes.byref(p), ctypes.byref(n))
                if p.value is not None or n.value != 0:
                    errors.append((k, it, "reset", p.value, n.value))
        L.chela_set_workspace(None, 0)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors[:5]
    # the main thread never set one
    p, n = ctypes.c_void_p(), ctypes.c_size_t()
    assert L.chela_get_workspace(ctypes.byref(p), ctypes.byref(n)) == 0 and p.value is None and n.value == 0


def test_set_workspace_alignment(L):
    assert L.chela_set_workspace(ctypes.c_void_p(0x1001), 1024) == -5
    assert L.chela_set_workspace(None, 0) == 0


def test_shutdown_is_idempotent(L):
    L.chela_shutdown()
    L.chela_shutdown()


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2406_08128_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.delenv("CHELA_LIB", raising=False)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()


def test_gated_argument_errors(L):
    f, z = L.chela_linattn_fwd_gated, L.chela_linattn_zfwd_gated
    Q, K, V, G, O, Y, SV = (A + i * SZ for i in range(7))
    dims = (1, 1, 64, 64, 64, 64, None)
    assert f(None, K, V, G, O, Y, SV, 1e-5, *dims) == -1
    assert f(Q, K, V, None, O, Y, SV, 1e-5, *dims) == -1
    assert f(Q, K, V, G, O, None, SV, 1e-5, *dims) == -1              # Y is required, O and saved are not
    assert f(Q, K, V, G, O, Y, SV, -1.0, *dims) == -2
    assert f(Q, K, V, G, O, Y, SV, float("nan"), *dims) == -2
    assert f(Q, K, V, G, O, Y, SV, float("inf"), *dims) == -2
    assert f(Q, K, V, G, O, Y + 4, SV, 1e-5, *dims) == -5
    assert f(Q, K, V, G, O, G, SV, 1e-5, *dims) == -6                 # Y on top of the gate
    assert f(Q, K, V, G, Y, Y, SV, 1e-5, *dims) == -6                 # O and Y are two outputs
    assert f(Q, K, V, G, O, Y, V, 1e-5, *dims) == -6                  # saved states over V
    assert f(Q, K, V, G, O, Y, SV, 1e-5, 1, 1, 64, 64, 96, 64, None) == -3
    assert f(Q, K, V, G, O, Y, SV, 1e-5, 1, 1, 64, 64, 64, 5, None) == -4
    assert f(None, None, None, None, None, None, None, 1e-5, 0, 1, 64, 64, 64, 64, None) == 0
    AF = A + 7 * SZ
    assert z(Q, None, V, G, O, Y, SV, 1e-5, *dims) == -1
    assert z(Q, AF + 4, V, G, O, Y, SV, 1e-5, *dims) == -5
    assert z(Q, AF, V, G, O, AF, SV, 1e-5, *dims) == -6
    assert z(Q, AF, V, G, O, Y, SV, -0.5, *dims) == -2
    assert z(None, None, None, None, None, None, None, 0.0, 1, 1, 0, 64, 64, 64, None) == 0


def test_gate_norm_argument_errors(L):
    f, g = L.chela_gate_norm_fwd, L.chela_gate_norm_bwd
    O, G, dY, dO, dG = (A + i * SZ for i in range(5))
    assert f(None, G, dO, 1e-5, 10, 64, None) == -1
    assert f(O, G, None, 1e-5, 10, 64, None) == -1
    assert f(O, G, dO, 1e-5, -1, 64, None) == -2
    assert f(O, G, dO, -1e-5, 10, 64, None) == -2
    assert f(O, G, dO, 1e-5, 10, 32, None) == -3
    assert f(O, G, dO + 2, 1e-5, 10, 64, None) == -5
    assert f(O, G, O, 1e-5, 10, 64, None) == -6
    assert f(O, G, O + 64, 1e-5, 10, 64, None) == -6
    assert f(None, None, None, 1e-5, 0, 64, None) == 0
    assert g(O, G, None, dO, dG, 1e-5, 10, 64, None) == -1
    assert g(O, G, dY, dO, None, 1e-5, 10, 64, None) == -1
    assert g(O, G, dY, dO, dO, 1e-5, 10, 64, None) == -6
    assert g(O, G, dY, G, dG, 1e-5, 10, 64, None) == -6
    assert g(O, G, dY, dY + 16, dG, 1e-5, 10, 64, None) == -6       # shifted overlap with dY is not the in-place case
    assert g(O, G, dY, dO, dY, 1e-5, 10, 64, None) == -6            # only dO may sit on dY
    assert g(O, G, dY, dO, dG, 1e-5, 10, 256, None) == -3
    assert g(None, None, None, None, None, 1e-5, 0, 128, None) == 0


def test_stream_probe_argument_errors(L):
    f = L.chela_stream_probe
    vp = ctypes.c_void_p
    ins = (vp * 4)(A, A + SZ, A + 2 * SZ, A + 3 * SZ)
    outs = (vp * 3)(A + 4 * SZ, A + 5 * SZ, A + 6 * SZ)
    assert f(ins, 0, outs, 3, 1024, None) == -2
    assert f(ins, 5, outs, 3, 1024, None) == -2
    assert f(ins, 4, outs, -1, 1024, None) == -2          # (0 outputs is a read-only mix: allowed)
    assert f(ins, 4, outs, 5, 1024, None) == -2
    assert f(ins, 4, outs, 3, 0, None) == 0
    assert f(None, 4, outs, 3, 1024, None) == -1
    assert f(ins, 4, outs, 3, 1000, None) == -5
    assert f((vp * 1)(None), 1, outs, 1, 1024, None) == -1
    assert f((vp * 1)(A + 4), 1, outs, 1, 1024, None) == -5
    assert f(ins, 4, (vp * 2)(A + 4 * SZ, A + 4 * SZ + 512), 2, 1024, None) == -6
    assert f(ins, 4, (vp * 1)(A + SZ), 1, 1024, None) == -6


def test_step_gated_argument_errors(L):
    f = L.chela_linattn_step_gated
    q, k, v, g, S, y = (A + i * SZ for i in range(6))
    assert f(q, k, v, None, S, y, 1e-5, 1, 1, 64, 64, None) == -1
    assert f(q, k, v, g, None, y, 1e-5, 1, 1, 64, 64, None) == -1
    assert f(q, k, v, g, S, y, -1.0, 1, 1, 64, 64, None) == -2
    assert f(q, k, v, g, S, y, 1e-5, 1, 1, 64, 96, None) == -3
    assert f(q, k, v, g + 2, S, y, 1e-5, 1, 1, 64, 64, None) == -5
    assert f(q, k, v, g, S, g, 1e-5, 1, 1, 64, 64, None) == -6
    assert f(q, k, v, g, g, y, 1e-5, 1, 1, 64, 64, None) == -6
    assert f(None, None, None, None, None, None, 1e-5, 0, 4, 64, 64, None) == 0


def test_noncausal_gated_argument_errors(L):
    f = L.chela_linattn_noncausal_fwd_gated
    Q, K, V, G, O, Y = (A + i * SZ for i in range(6))
    assert f(Q, K, V, None, O, Y, 1e-5, 1, 1, 64, 64, 64, None) == -1
    assert f(Q, K, V, G, O, None, 1e-5, 1, 1, 64, 64, 64, None) == -1
    assert f(Q, K, V, G, None, Y + 8, 1e-5, 1, 1, 64, 64, 64, None) == -5
    assert f(Q, K, V, G, Y, Y, 1e-5, 1, 1, 64, 64, 64, None) == -6
    assert f(Q, K, V, G, O, Q, 1e-5, 1, 1, 64, 64, 64, None) == -6
    assert f(Q, K, V, G, O, Y, float("nan"), 1, 1, 64, 64, 64, None) == -2
    assert f(Q, K, V, G, O, Y, 1e-5, 1, 1, 64, 64, 100, None) == -3
    assert f(None, None, None, None, None, None, 1e-5, 1, 0, 64, 64, 64, None) == 0
