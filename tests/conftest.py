import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Measured parity errors: for every test function the worst case of its comparisons against the oracle,
    as a fraction of the tolerance it was held to."""
    try:
        import util
    except Exception:
        return
    if not util.MEASURED:
        return
    worst = {}
    for test, what, err, tol in util.MEASURED:
        # named comparisons of the network-level tests are listed one by one, the others by their test function
        key = test if what else test.split("[")[0]
        if what:
            key = test + " :: " + what
        n, e, t, w = worst.get(key, (0, -1.0, 1.0, ""))
        if t <= 0 or err / max(tol, 1e-300) > e / max(t, 1e-300) or n == 0:
            e, t, w = err, tol, ("" if what else test[len(key):])
        worst[key] = (n + 1, e, t, w)
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("measured parity errors (worst comparison per test function: error / tolerance, comparisons, case)")
    for key in sorted(worst):
        n, e, t, w = worst[key]
        tr.write_line("  %-110s %.3e / %.1e = %4.2f  n=%-3d %s" % (key, e, t, e / t if t > 0 else float("inf"), n, w))
