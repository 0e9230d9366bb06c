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


def pytest_terminal_summary(terminalreporter):
    """Largest value errors that the GPU parity harness has seen, per kind of comparison."""
    mod = sys.modules.get("harness")
    lines = mod.Stats.lines() if mod is not None else []
    if lines:
        terminalreporter.write_sep("-", "largest errors against the oracle (relative to the bounds' scale)")
        for line in lines:
            terminalreporter.write_line(line)
