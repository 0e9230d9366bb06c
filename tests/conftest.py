import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a 'key: numbers' fixture (rows of a matrix separated by ';')."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":", 1)
            rows = [[float(x) for x in row.split()] for row in val.split(";")]
            out[key.strip()] = rows if len(rows) > 1 else rows[0]
    return out


@pytest.fixture(scope="session")
def worked_example():
    return load_golden("worked_example_m2n2t1.txt")
