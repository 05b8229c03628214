import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """A parity run must check against the oracle as committed: ZPP_ORACLE_LIB (which lets the
    mutant test load a deliberately broken build) may not be set when GPU tests are selected."""
    if any(item.get_closest_marker("gpu") for item in items) and os.environ.get("ZPP_ORACLE_LIB"):
        raise pytest.UsageError("ZPP_ORACLE_LIB is set: GPU parity tests would not run against the committed oracle")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
