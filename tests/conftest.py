import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the HIP library)")


def pytest_collection_modifyitems(config, items):
    # GPU tests announce themselves (and flush) before they start, so that a run
    # cut short by a device fault still names the case.
    pass


@pytest.fixture(autouse=True)
def _announce(request):
    if request.node.get_closest_marker("gpu"):
        print("\n[gpu-case] %s" % request.node.nodeid, flush=True)
    yield
