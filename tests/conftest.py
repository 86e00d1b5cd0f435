import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the library that is built, unless it was built from other sources than
    # the ones in the tree (content hash): then it is rebuilt first (hipcc cross-compiles
    # without a GPU), so an edited kernel is never tested against an older binary.
    from paper_2502_00425_amd import build as hip_build
    hip_build.ensure_fresh()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
