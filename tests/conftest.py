import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # A run that asks for the GPU tests (-m gpu) on a box where no GPU is visible is an error of
    # the run, not a green result with everything skipped.  A run that did not ask for them
    # (no -m, or -m "not gpu") just skips what it cannot execute.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    wanted = (config.getoption("-m") or "").replace("not gpu", "")
    if "gpu" in wanted:
        raise pytest.UsageError("-m gpu was requested but no GPU is visible to torch: the GPU tests cannot run here")
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
