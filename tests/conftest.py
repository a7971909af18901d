import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # the tests load what is built; only if nothing is there do they build it themselves
    from paper_2404_02015_amd import build as b

    if not os.path.exists(b.OUT) or not os.path.exists(b.DEMO):
        b.build(verbose=False)


@pytest.fixture(scope="session")
def oracle():
    from oracle import mux_oracle

    mux_oracle.build()
    return mux_oracle
