import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_params():
    """N = 16, three 20-bit chain primes in two digits (2 + 1, ragged), two special primes:
    small enough for exact big-integer checks."""
    from workloads.params import make_params
    return make_params(4, 3, 2, 2, bits=20)


@pytest.fixture(scope="session")
def cfg1_params():
    from workloads.params import CONFIGS
    return CONFIGS["cfg1_single_conv"].params()
