import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--oracle-lib", default=None,
                     help="shared object to load the CPU oracle from (the mutation test passes "
                          "deliberately broken builds; GPU tests refuse it)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    variant = config.getoption("--oracle-lib")
    if variant:
        import oracle
        oracle.use_library(variant)


def pytest_collection_modifyitems(config, items):
    if config.getoption("--oracle-lib"):
        for item in items:
            if item.get_closest_marker("gpu"):
                item.add_marker(pytest.mark.skip(reason="parity tests run against the committed oracle only"))


@pytest.fixture(scope="session")
def orc(request):
    import oracle
    if not request.config.getoption("--oracle-lib"):
        oracle.build(force=False)
    return oracle


@pytest.fixture(scope="session")
def gen():
    import synth
    synth.build_host(force=False)
    return synth
