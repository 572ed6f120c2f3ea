import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The ctypes binding over the built C-ABI library (fails loudly when it is not built)."""
    import paper_2605_17613_amd as vc
    vc.load()
    return vc


@pytest.fixture
def tunables(lib):
    """Set launch-shape tunables of the library for one test; every one is back at its default afterwards."""
    class _Tun:
        def __init__(self):
            self.names = set()

        def set(self, name, value):
            self.names.add(name)
            lib.vc_set_tunable(name, int(value))

    t = _Tun()
    yield t
    for name in t.names:
        lib.vc_set_tunable(name, -1)
