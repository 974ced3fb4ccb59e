import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _native_libraries():
    """Load what is built; rebuild what is missing or older than its sources (a hash of the
    sources and flags is kept beside each library), so that a test never runs a stale binary.
    hipcc cross-compiles without a GPU."""
    from paper_2406_02613_amd import build as acco_build
    from synth import build as synth_build
    if not acco_build.is_current():
        acco_build.build_acco()
    if not synth_build.device_current():
        synth_build.build_device()
    yield


@pytest.fixture(scope="session", autouse=True)
def _oracle_threads():
    """Let the oracle use the cores this process may run on (results do not depend on it)."""
    import oracle
    oracle.set_threads(min(oracle.usable_cores(), 16))
    yield
