import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")
    # the tests load the library that is built; only when none is there do they build it
    if not os.path.exists(os.path.join(ROOT, "paper_2605_06221_amd", "libuniprefill.so")):
        import __graft_entry__
        __graft_entry__.build()


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) when no device is visible."""
    has_gpu = None
    for item in items:
        if "gpu" in item.keywords:
            if has_gpu is None:
                import torch
                has_gpu = torch.cuda.is_available()
            if not has_gpu:
                item.add_marker(pytest.mark.skip(reason="no GPU visible"))
