import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs on the GPU box only)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: 'key = value  # citation' lines."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = [s.strip() for s in line.split("=", 1)]
            out[k] = float(v)
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden("paper_values.txt")


@pytest.fixture(scope="session")
def oracle_dict():
    import oracle
    return oracle.Dictionary()
