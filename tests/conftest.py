import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _oracle_threads():
    """Let the oracle use the cores this process may run on (results do not depend on it)."""
    import oracle
    oracle.set_threads(min(oracle.usable_cores(), 16))
    yield
