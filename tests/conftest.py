import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--oracle-lib", default=None,
                     help="load this build of the CPU oracle instead of oracle/libcombo_ref.so "
                          "(the mutation tests run the pins against deliberately wrong copies)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ref(request):
    """The CPU oracle (built on first use if the shared object is absent)."""
    from oracle import ref as _ref
    _ref.lib(request.config.getoption("--oracle-lib"))
    return _ref
