import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def orc():
    """The CPU oracle's Python wrapper (built on demand with gcc)."""
    from oracle import build as oracle_build
    oracle_build.build_oracle()
    from oracle import tutti_oracle
    tutti_oracle.lib()
    return tutti_oracle
