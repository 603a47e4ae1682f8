import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a whitespace-separated 'key v0 v1 ...' text fixture into a dict of
    string lists (comment lines start with '#')."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            out.setdefault(parts[0], []).append(parts[1:])
    return out


@pytest.fixture(scope="session")
def golden_dir():
    return GOLDEN


@pytest.fixture
def decode_override():
    """slim_decode_override for the duration of a test (host-side control of the decode launch geometry);
    the automatic choice is restored afterwards."""
    from paper_2410_09615_amd import binding as B
    yield B.slim_decode_override
    B.slim_decode_override("auto", 0)
