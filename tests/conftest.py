import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are only meaningful where a device is visible; without one they
    # are skipped loudly rather than silently passing on some fallback.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    # whole-schedule parity statistics (exact / excused / mismatch kept sets, max |dO|) of the GPU runs
    try:
        from tests import test_gpu_schedule as t
    except Exception:  # pragma: no cover
        return
    if t.PARITY_LOG:
        terminalreporter.write_sep("-", "device-vs-oracle parity statistics")
        for line in t.PARITY_LOG:
            terminalreporter.write_line(line)
