import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a golden text fixture: 'key: ints...' lines -> dict key -> list[int];
    lines without a key -> rows of ints under key '' ; '#' starts a comment."""
    out = {"": []}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if ":" in line:
                k, v = line.split(":", 1)
                out[k.strip()] = [int(x) for x in v.split()]
            else:
                out[""].append([int(x) for x in line.split()])
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
