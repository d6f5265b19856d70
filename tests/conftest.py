import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cnn():
    """The loaded GPU binding (builds the library first only if nothing is built)."""
    from paper_1602_06709_amd import binding
    binding.ensure_built()
    return binding
