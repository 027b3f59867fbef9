import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a `key: v v | v v` text fixture under tests/golden/ into {key: list of rows of floats}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            out[key.strip()] = [[float(v) for v in row.split()] for row in rest.split("|")]
    return out


@pytest.fixture(scope="session")
def golden_w1():
    return read_golden("w1_remap_example.txt")
