import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no GPU is visible.
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session", autouse=True)
def _libraries_are_built():
    """Tests load the libraries that are built; whatever is missing is built once, in-tree, before the first test."""
    from paper_2411_19379_amd import build as b
    if not os.path.exists(b.LIB_PATH):
        b.build_library()
    if not os.path.exists(b.CACHE_LIB_PATH):
        b.build_prefix_cache()
