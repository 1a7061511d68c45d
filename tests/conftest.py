import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--quick-parity", action="store_true", default=False,
                     help="full-size GPU parity cases compare sampled rows only (default: every active row)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lora():
    """The Python binding over the C-ABI library; GPU tests fail loudly if the library is missing."""
    import paper_2511_22880_amd as pkg
    return pkg


@pytest.fixture(scope="session")
def quick_parity(request):
    return bool(request.config.getoption("--quick-parity"))
