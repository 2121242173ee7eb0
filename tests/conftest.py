import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_init_tables():
    """The paper's printed init tables (App. F listing) from tests/golden/init_tables.txt."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", "init_tables.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *vals = line.split()
            out[name] = np.array([float(v) for v in vals], dtype=np.float64)
    return out


@pytest.fixture(scope="session")
def init_tables():
    return load_init_tables()
