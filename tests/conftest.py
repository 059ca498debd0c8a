import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "full: full-size baseline configurations (subset of gpu; minutes, up to 140 GB of HBM)")


@pytest.fixture(scope="session")
def orc():
    import oracle
    oracle.build()
    return oracle
