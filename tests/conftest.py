import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def override():
    """Set a testing hook of the library (la_debug_override) for the duration of a test."""
    from paper_2402_02057_amd import binding
    keys = []

    def set_(key, value):
        binding.la_debug_override(key, value)
        keys.append(key)
    yield set_
    for key in keys:
        binding.la_debug_override(key, None)
