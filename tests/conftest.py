import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Worst observed error / allowed error of the network comparisons of this run (tests/parity.py)."""
    try:
        import parity
    except Exception:
        return
    if parity.WORST:
        terminalreporter.write_line("parity: worst observed error as a fraction of the bound: " +
                                    ", ".join(f"{k}={v:.3f}" for k, v in sorted(parity.WORST.items())))
