import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_capture = None


def pytest_configure(config):
    global _capture
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _capture = config.pluginmanager.getplugin("capturemanager")


def say(msg):
    """A progress line that reaches the terminal even while pytest captures output: the long GPU tests
    print one per stage (a step done, a tensor compared), so that a log shows how far a run got."""
    if _capture is not None:
        with _capture.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)


@pytest.fixture(scope="session")
def orc():
    from oracle import oracle
    oracle.build()
    assert oracle.fp_env_ok()
    return oracle
