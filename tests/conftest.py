import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; only if none is there, build it once
    lib = os.path.join(ROOT, "paper_2504_06443_amd", "libspmm_brick.so")
    if not os.path.exists(lib):
        from paper_2504_06443_amd.build import build_library
        build_library(verbose=False)


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
