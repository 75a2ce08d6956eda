import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def rng():
    import numpy as np
    return np.random.default_rng(12345)


def pytest_terminal_summary(terminalreporter):
    """Worst value of each parity measure over the session (tests/parity.py collects them), per I/O dtype."""
    try:
        import parity
    except ImportError:
        return
    if not parity.STATS:
        return
    terminalreporter.write_line("parity summary (worst over %d comparisons against the oracle):" % len(parity.STATS))
    for dt in ("f32", "bf16"):
        rows = [s for s in parity.STATS if s[1] == dt]
        if not rows:
            continue
        w, g, r = (max(rows, key=lambda s: s[i]) for i in (2, 3, 4))
        terminalreporter.write_line("  %-4s whole tensor %.3e (%s)   worst (b,h) %.3e (%s)   worst row %.3e (%s)   [%d]"
                                    % (dt, w[2], w[0], g[3], g[0], r[4], r[0], len(rows)))
