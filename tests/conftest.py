import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' comments, then 'key v v v ...'."""
    import numpy as np
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            vals = [float(x) for x in parts[1:]]
            out[parts[0]] = vals
    n, d = int(out["n"][0]), int(out["d"][0])
    res = {"n": n, "d": d, "lambda": out["lambda"][0]}
    for k in ("Q", "K", "V", "dO", "O", "dQ", "dK", "dV"):
        res[k] = np.array(out[k], dtype=np.float64).reshape(1, 1, n, d)
    return res


@pytest.fixture
def golden():
    return load_golden
