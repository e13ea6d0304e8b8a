import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built; only if none is there do they build it (hipcc cross-compiles
    gfx950 without a GPU).  The binding itself never builds and never falls back."""
    from paper_2505_21070_amd import build
    build.ensure_built()


@pytest.fixture(scope="session")
def oracle_built():
    from oracle import build
    build.build()
    return True
