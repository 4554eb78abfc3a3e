import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import pbs_oracle
    pbs_oracle.build()
    return pbs_oracle


@pytest.fixture(scope="session")
def oracle_variants():
    from oracle import pbs_oracle_variants
    pbs_oracle_variants.build()
    return pbs_oracle_variants
