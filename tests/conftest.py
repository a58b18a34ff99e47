import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a 'key: v v v' text fixture under tests/golden/ (lines starting with # are comments)."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if ":" in line:
                k, v = line.split(":", 1)
                out[k.strip()] = [int(t) for t in v.split()]
            else:
                out.setdefault("rows", []).append([int(t) for t in line.split()])
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
