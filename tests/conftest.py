import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def pytest_terminal_summary(terminalreporter):
    import notes
    if notes.LINES:
        terminalreporter.section("coverage notes")
        for line in notes.LINES:
            terminalreporter.write_line(line)


@pytest.fixture(scope="session")
def oracle():
    from oracle import kdn_oracle
    kdn_oracle.build()
    return kdn_oracle


@pytest.fixture(scope="session", autouse=True)
def _library_present():
    """The library must match the sources beside it: a fresh checkout builds it once (hipcc
    cross-compiles without a GPU), a stale binary is built again, a failing build raises."""
    from paper_2409_13761_amd import build
    build.ensure_built()
