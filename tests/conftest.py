import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the library that is built; only when there is none do they build it
    # (hipcc cross-compiles without a GPU).
    from paper_2502_00425_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build(force=True)


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
