import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the in-tree library; it is compiled here only when none has been built yet.
    from paper_2508_04257_amd import build as kbuild

    if not os.path.exists(kbuild.LIB):
        kbuild.build(verbose=False)


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no device is visible.
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
