import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "timing: asserts a wall-clock window or a performance ordering (runs after the value checks)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    # Order of a run with -x: every comparison against the oracle first, then the tests that assert a
    # wall-clock window or a performance ordering (a noisy box must not hide parity results), and the
    # entry point that allocates nothing last (its file name already sorts last).
    def rank(item):
        if "test_zz_" in item.nodeid:
            return 2
        return 1 if "timing" in item.keywords else 0
    items.sort(key=rank)          # stable: the order inside each group stays as collected
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
