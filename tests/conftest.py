import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu)")


def read_golden_matrices(path):
    """Parse 'name rows cols v v v ...' lines (comments start with #)."""
    import numpy as np
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            name, rows, cols = parts[0], int(parts[1]), int(parts[2])
            vals = [float(v) for v in parts[3:]]
            assert len(vals) == rows * cols, name
            out[name] = np.array(vals, dtype=np.float64).reshape(rows, cols)
    return out


GOLDEN = os.path.join(ROOT, "tests", "golden")
