import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """A GPU parity run must compare against the real oracle: refuse to start one while the environment names a
    substitute oracle library (only the oracle mutation test's CPU child processes may use one)."""
    if os.environ.get("PE_ORACLE_LIB") and any(item.get_closest_marker("gpu") for item in items):
        raise pytest.UsageError("PE_ORACLE_LIB is set: GPU parity tests run against the built oracle only")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
