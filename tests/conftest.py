import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # tests that need the card are skipped on a machine without one
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this machine")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="module", autouse=True)
def _return_device_memory_after_each_module():
    """Hand cached device memory back to the driver when a test module is done.  The full-size modules hold up to
    138 GB; if that only went back at process exit, whatever runs on the card in the following ~20 s (measured: a
    benchmark process started right after a 138 GB process ends runs every sweep 3-4 % slower, one started 25 s later
    does not) would be measured against the driver's clean-up of that memory."""
    yield
    if "torch" in sys.modules:
        import gc
        import torch
        if torch.cuda.is_available():
            gc.collect()
            torch.cuda.empty_cache()
