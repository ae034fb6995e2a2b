import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: `NAME rows cols v...` lines, `#` comments."""
    import numpy as np

    out = {}
    path = os.path.join(ROOT, "tests", "golden", name)
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            r, c = int(tok[1]), int(tok[2])
            vals = np.array([float(v) for v in tok[3:]], dtype=np.float64)
            assert vals.size == r * c, (tok[0], vals.size, r, c)
            out[tok[0]] = vals.reshape(r, c)
    return out


@pytest.fixture(scope="session")
def golden_tiny():
    return load_golden("tiny_mdbf_worked.txt")
