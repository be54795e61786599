import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the HIP library)")
    config.addinivalue_line("markers", "sanitizer: builds the library with ASan + UBSan on its host code and re-runs the "
                                       "host-only tests against it in a child process (about a minute of compile time)")


def pytest_collection_modifyitems(config, items):
    # GPU tests call the HIP library; without a device they are skipped rather than failed.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
