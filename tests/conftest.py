import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden(name: str):
    """Values of one key of tests/golden/paper_values.txt as a list of ints."""
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    with open(path) as f:
        for line in f:
            parts = line.split()
            if parts and parts[0] == name:
                return [int(v) for v in parts[1:]]
    raise KeyError(name)
