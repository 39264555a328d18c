import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def dynb():
    """The ctypes binding of the HIP library; GPU tests fail loudly without it."""
    from paper_2305_12213_amd import binding
    binding.load()
    return binding
