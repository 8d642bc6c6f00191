import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """tests/golden/<name>: 'key value tol  # citation' lines -> {key: (value, tol)}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val, tol = line.split()
            out[key] = (float(val), float(tol))
    return out


@pytest.fixture(scope="session")
def paper_values():
    return load_golden("paper_values.txt")
