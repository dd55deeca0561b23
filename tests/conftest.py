import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: long-running full-size case")
    # the tests load the library that is built; it is rebuilt only if it is missing or was built from other sources
    # than the ones in the tree (hipcc cross-compiles without a GPU)
    from paper_2605_29346_amd import build as zg_build
    zg_build.ensure_current()


@pytest.fixture(scope="session")
def oracle():
    from oracle import zg_oracle
    zg_oracle.build()
    return zg_oracle
