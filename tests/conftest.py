import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Largest |gpu - oracle| seen per kind of comparison (tests/bars.py keeps the record)."""
    try:
        import bars
    except Exception:
        return
    if bars.observed:
        terminalreporter.write_line("largest deviations from the oracle in this run:")
        for label in sorted(bars.observed):
            terminalreporter.write_line(f"  {label}: {bars.observed[label]:.3e}")
