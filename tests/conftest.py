import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Tests load the library that is already built; only when none is there do they build it.
    lib = os.path.join(ROOT, "paper_2305_02299_amd", "libsrigl.so")
    if not os.path.exists(lib):
        from paper_2305_02299_amd_build import build_all
        build_all()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
