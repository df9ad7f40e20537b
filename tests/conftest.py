import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# The mutation test re-runs the pins against a deliberately broken copy of the oracle; that copy's
# parent directory is put in front so that `import oracle` finds it.
if os.environ.get("E4Q_TEST_ORACLE_PARENT"):
    sys.path.insert(0, os.environ["E4Q_TEST_ORACLE_PARENT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_lib():
    """The CPU oracle, compiled on first use if no built library is present."""
    import oracle

    oracle._load()
    return oracle
