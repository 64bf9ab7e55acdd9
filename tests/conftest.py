import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no GPU is visible.
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


@pytest.fixture
def say(request, capfd):
    """Progress lines of long GPU tests, printed past pytest's capture so that
    a run of several minutes is seen to be alive."""
    import time
    t0 = time.time()

    def emit(msg):
        with capfd.disabled():
            print(f"  [{request.node.name} +{time.time() - t0:5.1f}s] {msg}", flush=True)
    return emit
