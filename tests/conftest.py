import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture into {name: float64 ndarray}."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {}
    with open(path) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        key, r, c = lines[i].split()
        r, c = int(r), int(c)
        rows = [[float(x) for x in lines[i + 1 + k].split()] for k in range(r)]
        arr = np.array(rows, dtype=np.float64)
        assert arr.shape == (r, c), key
        out[key] = arr
        i += 1 + r
    return out


@pytest.fixture(scope="session")
def golden_1d():
    return load_golden("example_1d.txt")


@pytest.fixture(scope="session")
def golden_3x3():
    return load_golden("example_3x3.txt")
