import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The ctypes binding of the HIP library; GPU tests fail loudly when the
    shared object is missing rather than falling back to anything."""
    from paper_2502_06643_amd import binding
    return binding
