import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cfg1():
    import synthetic_inputs as si
    return si.make_config(1)


@pytest.fixture(scope="session")
def cfg2_small():
    """Config 2's automaton (256 states) with a reduced vocabulary."""
    import synthetic_inputs as si
    return si.make_config(2, V=6000)
