import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: full-size case (seconds on the GPU, minutes of oracle work where it is not precomputed)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as O
    O.build()
    return O
