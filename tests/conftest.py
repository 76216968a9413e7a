import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


@pytest.fixture(scope="session")
def rng_seed():
    return 20240711


@pytest.fixture(scope="session")
def lib():
    """The loaded C-ABI library; built first if the tree holds no build yet (hipcc
    cross-compiles without a GPU)."""
    import paper_2407_11550_amd as adakv
    if not os.path.exists(adakv.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return adakv.load_library()
