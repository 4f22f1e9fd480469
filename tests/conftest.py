import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, when no device is visible."""
    try:
        import torch
        have = torch.cuda.is_available()
    except Exception:
        have = False
    if have:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_runtest_logreport(report):
    """One line per finished GPU test into gpurun_out/test_progress.log: a run whose stdout is captured or buffered
    still shows that it is moving (the line is written when the test's call phase ends, never by a timer)."""
    if report.when != "call" or "gpu" not in report.keywords:
        return
    try:
        d = os.path.join(ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(f"{report.nodeid} {report.outcome} {report.duration:.1f}s\n")
    except OSError:
        pass
