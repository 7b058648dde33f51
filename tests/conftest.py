import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# tests/test_oracle_mutations.py runs the pins against a patched copy of the oracle: a directory
# that holds an `oracle/` folder of its own and comes first on the path
if os.environ.get("MRF_ORACLE_UNDER_TEST"):
    sys.path.insert(0, os.environ["MRF_ORACLE_UNDER_TEST"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import mrf_oracle
    mrf_oracle.build()
    return mrf_oracle
