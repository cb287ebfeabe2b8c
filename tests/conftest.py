import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    import oracle
    if not oracle._LIB_OVERRIDE:
        oracle.build(force=False)
    return oracle


@pytest.fixture(scope="session")
def gen():
    import synth
    synth.build_host(force=False)
    return synth
