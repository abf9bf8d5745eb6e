import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu)")
    import __graft_entry__
    __graft_entry__.ensure_built()   # loads what is built; compiles only if a library is missing altogether


@pytest.fixture(scope="session")
def oracle():
    import oracle as _o
    _o.lib()
    _o.set_threads(min(8, _o.max_threads()))
    return _o
