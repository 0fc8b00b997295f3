import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_kv(name):
    """Parse a golden 'key value' text fixture (lines starting with # are citations)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            out[k] = int(v)
    return out


def read_table1():
    rows = []
    with open(os.path.join(GOLDEN, "table1_adapter_sparsity.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, mx, avg, s = line.split()
            rows.append((name, int(mx), float(avg), float(s)))
    return rows


@pytest.fixture(scope="session")
def golden_fig3():
    return read_kv("fig3_virtual_tensor.txt")


@pytest.fixture(scope="session")
def golden_fig4():
    return read_kv("fig4_batched_rerouting.txt")


@pytest.fixture(scope="session")
def golden_table1():
    return read_table1()
