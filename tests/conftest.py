import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_available():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Worst row-scaled error per stage seen by the GPU parity harness in this session (empty without a GPU)."""
    harness = sys.modules.get("gpu_harness")
    if harness is None or not getattr(harness, "WORST", None):
        return
    terminalreporter.write_line("worst row-scaled error against the oracle, per stage (asserted tolerance):")
    for (what, dtype), err in sorted(harness.WORST.items()):
        tol = 1.0 if what.endswith("/ bound") else harness.TOL[dtype]
        terminalreporter.write_line("  %-40s %-5s %.3e  (%.3e)" % (what, dtype, err, tol))
    terminalreporter.write_line("largest top-2 margin at which a hash digit took the runner-up vertex: %.3e (accepted below %.0e)"
                                % (harness.WORST_FLIP_MARGIN[0], harness.TIE_MARGIN))
