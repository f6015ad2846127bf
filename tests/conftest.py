import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(scope="session")
def small_oracle():
    """N=2^6, three 30-bit primes, dnum 3 (alpha 1), noise on."""
    from oracle import Oracle
    o = Oracle(6, [30, 30, 30], 3, 40, seed=7)
    o.keygen()
    return o
