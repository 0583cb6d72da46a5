import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import kdn_oracle
    kdn_oracle.build()
    return kdn_oracle


@pytest.fixture(scope="session", autouse=True)
def _library_present():
    """A fresh checkout holds no built library: build it once (hipcc cross-compiles without a
    GPU).  A library that is there is used as it is."""
    from paper_2409_13761_amd import build
    build.ensure_built()
