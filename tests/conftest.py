import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # pytest-timeout registers this mark itself when it is installed; without it the mark is inert
    config.addinivalue_line("markers", "timeout(seconds): time limit of a test (pytest-timeout)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped (not failed) when no device is present and they were not
    # deselected with -m "not gpu".
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
