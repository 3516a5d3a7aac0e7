import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# test_oracle_mutants.py runs the pin files against a changed COPY of oracle/: the copy's parent directory goes first
if os.environ.get("NETMAX_TEST_ORACLE_ROOT"):
    sys.path.insert(0, os.environ["NETMAX_TEST_ORACLE_ROOT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ora():
    import oracle
    oracle.lib()
    return oracle
