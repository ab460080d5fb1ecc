import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: 'key v v v' lines, '/' separates matrix rows."""
    import numpy as np

    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(None, 1)
            rows = [[float(v) for v in row.split()] for row in rest.split("/")]
            a = np.array(rows, dtype=np.float64)
            out[key] = a[0, 0] if a.size == 1 else (a[0] if len(rows) == 1 else a)
    return out


@pytest.fixture(scope="session")
def oracle():
    import oracle as o

    o.build()
    return o
