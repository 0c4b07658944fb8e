import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the in-tree library; when nothing is built yet (a fresh checkout), build it once
    from paper_2412_05270_amd import build, library_path
    if not os.path.exists(library_path()):
        build.build(verbose=False)


def read_golden(name):
    """Parse a golden text file: '#' lines are comments/citations, others 'key: value'."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            out[key.strip()] = val.strip()
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
