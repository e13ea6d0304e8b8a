import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built; only if none is there (or a source is newer than it) do they
    build it (hipcc cross-compiles gfx950 without a GPU).  The binding itself never builds and never falls back."""
    from paper_2505_21070_amd import build
    build.ensure_built()


@pytest.hookimpl(tryfirst=True)
def pytest_runtest_setup(item):
    """Names every GPU test on the real stderr before it starts, so that a run which dies inside a kernel
    still says which case it was in, and a long run keeps printing."""
    if item.get_closest_marker("gpu") is None:
        return
    capman = item.config.pluginmanager.getplugin("capturemanager")
    if capman is not None:
        with capman.global_and_fixture_disabled():
            sys.stderr.write(f"\n[gpu test] {item.nodeid}\n")
            sys.stderr.flush()


@pytest.fixture
def progress(request):
    """progress("text"): one flushed line on the real stderr from inside a long test."""
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def say(msg):
        with capman.global_and_fixture_disabled():
            sys.stderr.write(f"  [{request.node.name}] {msg}\n")
            sys.stderr.flush()
    return say


@pytest.fixture(scope="session")
def oracle_built():
    from oracle import build
    build.build()
    return True
