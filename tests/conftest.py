import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built in-tree; it is compiled here only when there is none."""
    from paper_2605_18739_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build(verbose=False)


@pytest.fixture(scope="session")
def oracle():
    from oracle import nvfp4_oracle
    nvfp4_oracle.build()
    return nvfp4_oracle
