import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # load what is built if it matches the sources; otherwise compile (hipcc cross-compiles
    # without a GPU)
    from paper_2402_10876_amd import build
    build.ensure_built()


def pytest_report_header(config):
    from paper_2402_10876_amd import build
    return "libtwgemm: " + build.describe()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
