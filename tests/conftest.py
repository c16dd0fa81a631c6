import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import sik_oracle
    # OpenMP over (batch, head) on the cores this process may use (the loops inside one head stay serial)
    sik_oracle.set_threads(min(16, len(os.sched_getaffinity(0))))
    return sik_oracle
