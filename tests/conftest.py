import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # compile a missing or stale oracle now, before any test initialises the GPU: a process that
    # has done so must not start compiler child processes
    import oracle
    oracle.build()


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    return oracle
