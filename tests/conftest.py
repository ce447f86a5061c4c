import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_available() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    # A GPU test on a box without a GPU is a configuration error of the run,
    # not a pass: skip it loudly so it can never count as green.
    if _gpu_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible (gpu-marked test)")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)
