import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _native_helpers():
    """Build the CPU-side helper libraries (input generator, oracle) when they are absent."""
    import oracle
    import workloads

    if not os.path.exists(os.path.join(ROOT, "workloads", "libworkloads.so")):
        workloads.build()
    if not os.path.exists(os.path.join(ROOT, "oracle", "liboracle.so")):
        oracle.build()
    yield
