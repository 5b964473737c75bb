import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import oracle as orc
    orc.build()
    return orc


def pytest_terminal_summary(terminalreporter):
    """What the oracle comparisons of this run saw, beside their pass/fail."""
    from tests.parity import TOTAL
    if TOTAL.queries:
        terminalreporter.write_line(f"oracle comparisons: {TOTAL.summary()}")
