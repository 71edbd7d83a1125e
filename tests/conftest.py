import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse tests/golden/<name>: 'key = values', matrix rows separated by ';'."""
    import numpy as np
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = (s.strip() for s in line.split("=", 1))
            if key == "loss":
                out[key] = val
                continue
            rows = [[float(v) for v in row.split()] for row in val.split(";")]
            arr = np.array(rows, dtype=np.float64)
            out[key] = arr[0, 0] if arr.size == 1 and key in (
                "d", "K", "T", "D", "eps", "regret", "bound", "delta", "eta") else (arr[0] if len(rows) == 1 else arr)
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
