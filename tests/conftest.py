import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# every workspace the binding allocates in a test starts as 0xFF bytes (NaN, -1), so that a kernel that reads a
# section before anything has written it cannot pass by finding the values an earlier call left there
os.environ.setdefault("POLLUX_POISON_WORKSPACE", "1")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """Skip GPU tests cleanly where no device is visible (they are selected with -m gpu where a device is present)."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
