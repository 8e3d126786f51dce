import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    import __graft_entry__
    __graft_entry__.ensure_built()          # tests load the built library; compile only if there is none


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o
