import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The oracle's library is loaded here (and compiled first if it is missing: a child process), before
    # the check below or any test touches the GPU; a process that has done that starts no other programs.
    from oracle import model
    model.load()


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(params=["table", "driver"])
def pool_mode(request):
    """Runs a GPU test twice: on a plain pool read through the software table, and on a driver-mapped
    pool whose kernels read each tensor as a contiguous virtual address range (the paper's mechanism)."""
    from tests import gpu_harness as H
    H.POOL_MODE = request.param
    yield request.param
    H.POOL_MODE = "table"
