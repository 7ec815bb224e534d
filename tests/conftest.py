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
    """Parse a 'key value...' text fixture: returns (dict of scalar keys, list of numeric rows)."""
    scalars, rows = {}, []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            try:
                float(parts[0])
                rows.append([float(p) for p in parts])
            except ValueError:
                scalars[parts[0]] = float(parts[1])
    return scalars, rows


@pytest.fixture(scope="session")
def golden():
    return read_golden
