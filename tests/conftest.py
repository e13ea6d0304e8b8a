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


def pytest_sessionfinish(session, exitstatus):
    """DP_PARITY_REPORT=<file>: every GPU-vs-oracle comparison of the session (max-abs, max-rel, relative L2 of the
    whole tensor and of the worst row) as JSON lines, plus a summary per storage type on stderr."""
    path = os.environ.get("DP_PARITY_REPORT")
    if not path:
        return
    import json
    try:
        from harness import REPORT
    except ImportError:
        return
    with open(path, "w") as f:
        for r in REPORT:
            f.write(json.dumps(r) + "\n")
    for dt in ("f32", "bf16"):
        rows = [r for r in REPORT if r["dtype"] == dt]
        if rows:
            sys.stderr.write(f"[parity report] {dt}: {len(rows)} comparisons, worst max_abs {max(r['max_abs'] for r in rows):.3e}, "
                             f"worst whole-tensor rel L2 {max(r['rel_l2'] for r in rows):.3e}, "
                             f"worst single-row rel L2 {max(r['worst_row'] for r in rows):.3e}\n")
