import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    import progress
    progress.capman = config.pluginmanager.getplugin("capturemanager")


@pytest.fixture(autouse=True)
def _name_the_running_test(request):
    """Long runs name the test they are in now and then (see progress.py)."""
    import progress
    progress.tick(f"[{request.node.nodeid}]", every=30.0)
    yield
