import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def load_table(name):
    """Numeric columns (without the level index) of a text fixture under tests/golden/."""
    path = os.path.join(ROOT, "tests", "golden", name)
    rows = [[float(v) for v in ln.split()[1:]] for ln in open(path) if ln.strip() and not ln.startswith("#")]
    return np.array(rows, dtype=np.float64)


@pytest.fixture(scope="session")
def tables():
    return {"I64": load_table("table_codebooks_I64.txt"),
            "bof4s": load_table("table_bof4s_mse_blocksizes.txt"),
            "emp_theo": load_table("table_bof4_mse_emp_vs_theo_I64.txt")}
