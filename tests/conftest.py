import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def toy_keys():
    from oracle import tfhe
    return tfhe.keygen(tfhe.TOY, 190600148)


@pytest.fixture(scope="session")
def real_keys():
    from oracle import tfhe
    return tfhe.keygen(tfhe.REAL, 190600148)


@pytest.fixture(scope="session")
def section4_keys():
    """The ring degree of the paper's leveled setting (Section 4, "TFHE setting": N-bar = 2048) with a short TLWE key:
    the leveled operations use the ring key only, and a small n keeps the oracle's key generation cheap."""
    from oracle import tfhe
    return tfhe.keygen(tfhe.Params(n=16, N=2048), 190600148)
