import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden_path(name):
    return os.path.join(ROOT, "tests", "golden", name)


def read_golden(name):
    """Parse a golden text fixture: `key | values | citation` per line."""
    out = {}
    with open(golden_path(name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals, _cite = [s.strip() for s in line.split("|", 2)]
            out[key] = [float(v) for v in vals.split()]
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden("paper_values.txt")
