import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Numbers of a fixture under tests/golden/: '#' lines are comments (the citation)."""
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    rows = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":", 1)
            rows[key.strip()] = val.strip()
    return rows


@pytest.fixture(scope="session")
def golden():
    return load_golden
