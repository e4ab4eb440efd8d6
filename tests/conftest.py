import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_hand_cases():
    """{case: {(row, col): value}} from tests/golden/hand_cases.txt."""
    path = os.path.join(ROOT, "tests", "golden", "hand_cases.txt")
    cases = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, i, j, v = line.split()
            cases.setdefault(name, {})[(int(i), int(j))] = float(v)
    return cases
