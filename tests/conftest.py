import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def load_golden(name):
    """Parse tests/golden/<name>: 'key value [value ...]' lines, '#' comments."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, *v = line.split()
            vals = [float(t) for t in v]
            out[k] = vals[0] if len(vals) == 1 else vals
    return out


@pytest.fixture(scope="session")
def golden():
    return load_golden
