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


@pytest.fixture(params=["in_expansion", "by_rule"])
def value_path(request):
    """A fused step produces the new value row either inside its expansion pass
    or in the launch that appends the key row; the library picks by the size of the value bases.
    Tests of small cases run both ways."""
    from paper_2603_23914_amd import binding as ap
    ap.ap_set_fused_value_min_bytes(0 if request.param == "in_expansion" else -1)
    yield request.param
    ap.ap_set_fused_value_min_bytes(-1)


@pytest.fixture(scope="session")
def paper_values():
    return load_golden("paper_values.txt")
