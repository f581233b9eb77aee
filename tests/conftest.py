import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The libraries are built beforehand; build here only what is missing (a fresh checkout)."""
    from paper_2603_27138_amd import build
    if not os.path.exists(build.LIB) or not os.path.exists(build.CALIB_LIB):
        build.build()
    if not os.path.exists(build.HOST_LIB):
        build.build_host()


@pytest.fixture(scope="session")
def oracle_lib():
    import oracle
    oracle.build()
    return oracle


@pytest.fixture(autouse=True)
def _output_guards(request):
    """After every GPU test: no entry point wrote outside an output tensor of the test harness
    (tests/gpu_harness.Arena), also for the calls a test made on those tensors directly."""
    yield
    if request.node.get_closest_marker("gpu") is not None:
        from tests import gpu_harness
        gpu_harness.check_all_guards()
