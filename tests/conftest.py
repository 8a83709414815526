import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _hip_library():
    """The tests load the library that is built; only when there is none do they compile it."""
    from paper_2503_00245_amd import build as hip_build
    return hip_build.ensure_built()


@pytest.fixture(scope="session")
def oracle():
    from oracle import build as obuild
    obuild.build(force=False)
    from oracle import moe_oracle
    return moe_oracle
