import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; only a tree with none gets one compiled here (hipcc cross-compiles
    # for gfx950 without a GPU)
    from paper_2311_11514_amd.build import LIB as LIB_PATH, build_library
    if not os.path.exists(LIB_PATH):
        build_library()


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no device exists and they were not deselected
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
