import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs the HIP library through its C ABI)")


def read_golden_kv(name):
    """Parse a `key = value` golden file; integers may be decimal, 0x or 0b; floats allowed."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val = [t.strip() for t in line.split("=", 1)]
            try:
                out[key] = int(val, 0)
            except ValueError:
                out[key] = float(val)
    return out


@pytest.fixture(scope="session")
def paper_examples():
    return read_golden_kv("paper_examples.txt")
