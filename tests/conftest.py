import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU box)")


@pytest.fixture(scope="session")
def oracle_attn():
    """The fp64 C oracle, compiled on first use."""
    from oracle import attn
    attn.build()
    return attn


@pytest.fixture(scope="session")
def mepic():
    """The product binding; loading fails loudly when the HIP library has not been built."""
    import paper_2512_16822_amd as m
    m.load()
    return m
