import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_sessionstart(session):
    """The tests load the library that is built in-tree; only if there is none do they build it first
    (hipcc cross-compiles for gfx950 without a GPU).  The package itself never builds and never falls back."""
    import paper_1709_04057_amd as lr
    if not os.path.exists(lr.lib_path()):
        from paper_1709_04057_amd import build as _build
        _build.build()


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle
