import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def progress(request):
    """A print that is not held back by output capture: the long checker runs of the full-size tests report each
    completed step (a layer of the fp64 checker takes up to a minute), so a run that is merely busy shows it."""
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def say(msg: str) -> None:
        if capman is None:
            print(msg, flush=True)
            return
        with capman.global_and_fixture_disabled():
            print(msg, flush=True)
    return say
