import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # test modules import the binding at collection time: load what is built, compile only if
    # nothing is
    from paper_2511_12653_amd import build
    build.ensure_built()


@pytest.fixture(scope="session")
def oracle():
    from oracle import fq_oracle
    fq_oracle.lib()
    return fq_oracle
