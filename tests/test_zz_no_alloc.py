"""The entry point that allocates nothing (chela_linattn_fwd_noalloc) against chela_linattn_fwd, through the C ABI.

Two calls in a row on the library's fixed scratch array, the second on a smaller input, so that the second finds the
first one's states in the array.  The bar is the one of the other bf16 parity tests (rel-L2 <= 2e-2); the two entry
points run the same kernels on the same split, so the outputs are in fact expected to be identical bit for bit, and
both are also held against the fp64 oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2406_08128_amd import binding
from paper_2406_08128_amd.workloads import WORKLOADS, make_inputs, shrink, to_f64_numpy

pytestmark = pytest.mark.gpu

BAR = 2e-2


def _rel_l2(a, b):
    a, b = a.double(), b.double()
    return float((a - b).norm() / b.norm())


def _one_call(w, chunk=64):
    x = make_inputs(w, with_dO=False)
    d = {k: v.cuda() for k, v in x.items()}
    need = binding.chela_linattn_workspace_bytes(w.B, w.H, w.N, w.dk, w.dv, chunk, False, binding.DTYPE_BF16)
    print("\n   noalloc case B%d H%d N%d dk%d dv%d: %d bytes of states" % (w.B, w.H, w.N, w.dk, w.dv, need), flush=True)
    assert 0 < need <= (32 << 20), "the case is meant to use the scratch array"
    O = torch.full_like(d["V"], float("nan"))           # caller-owned output, allocated before the call
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.chela_linattn_fwd_noalloc(d["Q"], d["K"], d["V"], O, chunk=chunk)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before       # (torch's view: the binding allocated no tensor either)
    ref = binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], chunk=chunk)
    torch.cuda.synchronize()
    err = _rel_l2(O, ref)
    print("   rel-L2 against chela_linattn_fwd = %.3e, identical = %s" % (err, torch.equal(O, ref)), flush=True)
    assert np.isfinite(err) and err <= BAR
    assert torch.equal(O, ref), "same kernels, same split: the two entry points should agree bit for bit"
    Qn, Kn, Vn = (to_f64_numpy(x[n]) for n in "QKV")
    err_o = oracle.rel_l2(to_f64_numpy(O), oracle.fwd_recurrent(Qn, Kn, Vn))
    print("   rel-L2 against the oracle        = %.3e" % err_o, flush=True)
    assert np.isfinite(err_o) and err_o <= BAR


def test_noalloc_forward_twice_second_call_smaller():
    big = shrink(WORKLOADS["lm_bf16"], B=2, H=6, N=8192, seed=71)        # several segments per sequence
    small = shrink(WORKLOADS["lm_bf16"], B=1, H=3, N=3000, dk=64, dv=128, seed=72)   # ragged, another state shape
    _one_call(big)
    _one_call(small)


def test_noalloc_rejects_what_does_not_fit():
    # 149 long sequences with 128 x 128 states: the planner's split needs 46 MiB of segment states
    B, H, N, dk, dv = 1, 149, 1984972, 128, 128
    need = binding.chela_linattn_workspace_bytes(B, H, N, dk, dv, 64, False, binding.DTYPE_BF16)
    assert need > (32 << 20)
    L = binding.lib()
    a = 0x10000
    rc = L.chela_linattn_fwd_noalloc(a, a + (1 << 40), a + (2 << 40), a + (3 << 40), B, H, N, dk, dv, 64, None)
    assert rc == -7          # CHELA_ERR_WORKSPACE, before anything is enqueued or any pointer is touched
