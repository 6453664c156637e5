import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden text fixture: '#' comments, 'key = numbers' lines or bare rows."""
    path = os.path.join(ROOT, "tests", "golden", name)
    keyed, rows = {}, []
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if "=" in line:
                k, v = line.split("=", 1)
                keyed[k.strip()] = v.split()
            else:
                rows.append(line.split())
    return keyed, rows


@pytest.fixture(scope="session")
def golden():
    return read_golden
