import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.hookimpl(tryfirst=True)
def pytest_runtest_setup(item):
    """MA_ORACLE_LIBRARY swaps the checker for another build (the mutation tests do that on purpose, on
    the CPU).  A GPU parity test checked against anything but the committed oracle proves nothing."""
    if item.get_closest_marker("gpu") is not None and os.environ.get("MA_ORACLE_LIBRARY"):
        pytest.fail("MA_ORACLE_LIBRARY is set (%s): GPU parity tests run against the committed oracle only"
                    % os.environ["MA_ORACLE_LIBRARY"])


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
