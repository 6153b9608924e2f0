import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests never run silently on a box without a GPU: they are skipped
    # loudly there, and on a GPU machine they fail if the HIP library is missing.
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session", autouse=True)
def _libyoco_built():
    """Load the in-tree libyoco.so; build it first only if nothing is built yet."""
    from paper_2405_05254_amd import binding, build
    if not os.path.exists(binding.lib_path()):
        build.build_lib()
    yield
