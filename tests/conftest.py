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


def pytest_terminal_summary(terminalreporter):
    """Worst relative gradient error seen on elements with |oracle| >= 1 (the strict gate of the parity tests)."""
    try:
        import harness
    except Exception:
        return
    if harness.WORST_REL:
        terminalreporter.write_line("worst |hip - oracle| / |oracle| where |oracle| >= 1 (gate 1e-5):")
        for k, v in sorted(harness.WORST_REL.items(), key=lambda kv: -kv[1])[:12]:
            terminalreporter.write_line(f"  {k}: {v:.3e}")
