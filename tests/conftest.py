import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Worst per-row relative error each GPU parity test saw (rows measured on their own scale)."""
    from tests import util
    if not util.WORST_ROW_ERR:
        return
    terminalreporter.write_line("worst per-row relative error against the oracle, by test (largest first):")
    for test, err in sorted(util.WORST_ROW_ERR.items(), key=lambda kv: -kv[1])[:25]:
        terminalreporter.write_line(f"  {err:9.3e}  {test}")
