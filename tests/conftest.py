import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """Compile the C oracle (if it is missing or older than its source) before any test runs, so that no compiler
    is started from a process that has already initialised the GPU."""
    from oracle import ef21_oracle
    ef21_oracle.build()


@pytest.fixture(scope="session")
def oracle():
    from oracle import ef21_oracle
    ef21_oracle.build()
    return ef21_oracle
