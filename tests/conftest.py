import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """How close the GPU-vs-oracle comparisons came to their three bounds (tensor, row, element)."""
    try:
        import util
    except Exception:
        return
    if not util.WORST:
        return
    terminalreporter.write_line("worst fraction of the parity bounds (tensor / row / element):")
    for key in sorted(util.WORST):
        t, r, e = util.WORST[key]
        terminalreporter.write_line("  %-70s %.3f %.3f %.3f" % (key[:70], t, r, e))
