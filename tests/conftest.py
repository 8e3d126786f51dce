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


class _RefCache:
    """Oracle results of the full-size program-tree configurations, computed once per session
    (config 2 takes about 10 s on the 16 host cores of a GPU machine)."""

    def __init__(self, oracle):
        self.oracle = oracle
        self.items = {}

    def get(self, key, make):
        if key not in self.items:
            w = make()
            self.items[key] = (w, self.oracle.iep_forward_workload(w))
        return self.items[key]


@pytest.fixture(scope="session")
def full_refs(oracle):
    return _RefCache(oracle)
