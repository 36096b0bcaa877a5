import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path)")


@pytest.fixture(scope="session")
def hs():
    """The Python binding over the C-ABI library; GPU tests fail loudly if it is absent."""
    import paper_2402_04466_amd as pkg
    return pkg
