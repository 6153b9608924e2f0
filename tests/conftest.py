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
    """Load the in-tree libyoco.so. It is rebuilt first when it is missing or was built from other sources than the
    tree holds now (a hash of the sources is stored beside it), so the tests never describe a stale library."""
    from paper_2405_05254_amd import build
    if not build.is_current():
        build.build_lib()
    yield
