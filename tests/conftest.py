import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o


@pytest.fixture
def options():
    """Setter for the library's tuning switches; every switch is back at its default after the test."""
    from paper_2502_18394_amd import binding
    yield binding.set_option
    for which in range(7):
        binding.set_option(which, -1)
