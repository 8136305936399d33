import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden text fixture: 'key: v v v' lines and an optional 'W:' block."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {}
    rows = None
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line == "W:":
                rows = []
                out["W"] = rows
                continue
            if ":" in line:
                rows = None
                key, rest = line.split(":", 1)
                out[key.strip()] = [float(t) for t in rest.split()]
            elif rows is not None:
                rows.append([float(t) for t in line.split()])
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
