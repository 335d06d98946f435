import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    from oracle import oracle
    oracle.lib()
    return oracle


@pytest.fixture(scope="session")
def real_keys(orc):
    """Oracle keys at the benchmark parameters (n=500, N=1024, ...)."""
    import workloads
    return orc.Keys(orc.default_params(), workloads.KEY_SEED)


@pytest.fixture(scope="session")
def toy_keys(orc):
    """Small parameters at which the index-by-index product definition is affordable."""
    P = orc.Params(16, 64, 1, 2, 10, 8, 2, -15, -25)
    return orc.Keys(P, 4242)


@pytest.fixture
def say(request):
    """Progress lines of long GPU tests, written past pytest's capture: whoever watches the run sees
    each finished step of the work, not a silent process."""
    capture = request.config.pluginmanager.getplugin("capturemanager")

    def _say(msg):
        with capture.global_and_fixture_disabled():
            sys.stderr.write(msg + "\n")
            sys.stderr.flush()
    return _say


def pytest_runtest_logstart(nodeid, location):
    """One unbuffered line per test: long GPU tests must not look like a hung run to whoever
    watches the output through a pipe."""
    sys.stderr.write(f"[start] {nodeid}\n")
    sys.stderr.flush()
