"""MI355X-native causal linear attention (the hot path of CHELA, Sec. 4.1).

The compute lives in csrc/ (hand-written HIP for gfx950 behind a C ABI, see
include/chela.h); `binding` marshals torch tensors into that ABI.  Nothing is
loaded at import time; the first call loads libchela.so and fails loudly if it
has not been built.  There is no CPU fallback.
"""
from .workloads import WORKLOADS, Workload, make_inputs  # noqa: F401

__all__ = ["WORKLOADS", "Workload", "make_inputs", "binding", "workloads"]
