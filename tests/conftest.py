import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU harness)")


@pytest.fixture(scope="session")
def oracle_threads():
    """Use a few host threads for the oracle's outermost parallel index."""
    import oracle

    n = max(1, min(8, oracle.max_threads()))
    oracle.set_threads(n)
    return n
