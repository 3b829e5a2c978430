import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# tests/test_oracle_mutants.py runs the pins against deliberately broken copies of the oracle package:
# it names the directory that holds such a copy here, and that copy is then the one "import oracle" finds
if os.environ.get("REGOT_TEST_ORACLE_PATH"):
    sys.path.insert(0, os.environ["REGOT_TEST_ORACLE_PATH"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle._load()
    return oracle
