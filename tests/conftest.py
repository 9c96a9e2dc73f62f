import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs the HIP library)")


@pytest.fixture(scope="session")
def lib():
    """The ctypes binding; GPU tests fail loudly if the library is not built."""
    from paper_2104_04731_amd import binding
    binding.load()
    return binding
