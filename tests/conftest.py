import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def say(request):
    """Progress lines of long tests, written past pytest's output capture: a test that runs for minutes
    must not look hung to whoever watches the run."""
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def _say(*args):
        with capman.global_and_fixture_disabled():
            print(*args, flush=True)
    return _say
