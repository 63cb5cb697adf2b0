import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import lsm_oracle
    lsm_oracle.build()
    return lsm_oracle


@pytest.fixture
def say(capsys):
    """print() for the long tests: shown even when pytest captures output, so that a run of several minutes is not
    silent."""
    def say(*args):
        with capsys.disabled():
            print(*args, flush=True)
    return say
