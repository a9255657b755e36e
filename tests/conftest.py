import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C-ABI)")


def pytest_sessionstart(session):
    """The tests load the library that is built; only a tree in which nothing is built yet (a fresh
    clone) compiles it here first.  The product itself never does: its import fails without it."""
    from paper_2605_06472_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_06472_amd import build
        build.build()


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    return _oracle
