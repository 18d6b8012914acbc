import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load what is built; only when nothing is built do they build it themselves."""
    from paper_2407_15545_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build(force=True)
    if not os.path.exists(hip_build.TORCH_EXT):
        hip_build.build_torch_extension()


GOLDEN = os.path.join(ROOT, "tests", "golden")


def read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def golden():
    return read_table
