import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name: str) -> dict:
    """Parse a `key: ints` text fixture; a value containing '|' is a matrix (rows split on '|')."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            if "|" in val:
                out[key.strip()] = np.array([[float(t) for t in row.split()] for row in val.split("|")])
            else:
                out[key.strip()] = np.array([float(t) for t in val.split()])
    return out


@pytest.fixture(scope="session")
def example():
    return load_golden("worked_example_5x12.txt")
