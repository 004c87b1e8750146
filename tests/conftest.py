import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built in-tree; only if there is none do they build it
    (hipcc cross-compiles without a GPU)."""
    from paper_2209_10778_amd import binding, build
    if not os.path.exists(binding.lib_path()) and os.path.exists(build.HIPCC):
        build.build(verbose=False)


def pytest_collection_modifyitems(config, items):
    # GPU tests are only meaningful when selected explicitly with -m gpu on a GPU machine.
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
