import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; only a tree with none gets one built here
    import __graft_entry__

    __graft_entry__.ensure_built()


@pytest.fixture(scope="session")
def lib():
    """The HIP library binding; GPU tests fail loudly if it is not built."""
    import paper_2412_00099_amd as pkg

    return pkg
