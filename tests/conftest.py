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
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Largest |gpu - oracle| seen by the parity helpers in this session, per kind of tensor and storage type."""
    try:
        import fb_testlib
    except Exception:
        return
    if not fb_testlib.ACHIEVED:
        return
    terminalreporter.write_line("achieved max |gpu - oracle| (kind, dtype: max error, largest |oracle| value, comparisons)")
    for (kind, dtype), (e, m, n) in sorted(fb_testlib.ACHIEVED.items()):
        terminalreporter.write_line(f"  {kind:6s} {dtype:5s}: {e:.3e}   (|oracle| up to {m:.3g}, {n} comparisons)")
