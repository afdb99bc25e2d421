import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU box)")


import pytest


@pytest.fixture
def fx_opt():
    """Set switches of the library (fx_set_option) for one test; every one goes back to automatic afterwards."""
    import paper_2407_01781_amd as fx
    changed = []

    def set_(name, value):
        changed.append(name)
        fx.set_option(name, int(value))

    yield set_
    for name in changed:
        fx.set_option(name, -1)
