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
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(params=["two_steps", "one_step"])
def gradient_steps(request):
    """Both ways dvp_forward_backward has of writing the gradient, whatever the size of the matrix
    (by default the size decides: dvp_set_split_min_bytes in include/dvp.h)."""
    from paper_2512_23087_amd import dvp
    old = dvp.set_split_min_bytes(0 if request.param == "two_steps" else 2 ** 63 - 1)
    yield request.param
    dvp.set_split_min_bytes(old)
