import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_inputs():
    import workloads
    return workloads.generate(workloads.TINY)


@pytest.fixture(scope="session", autouse=True)
def built_library():
    """The C-ABI library, rebuilt when it is missing or older than the sources in the tree (before
    any test touches a GPU: the build runs hipcc as child processes)."""
    from paper_2605_02960_amd import build as moe_build
    return moe_build.ensure_built()
