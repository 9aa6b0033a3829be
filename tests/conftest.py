import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture into {section: [[float, ...], ...]}."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line[0].isalpha():
                cur = line
                out[cur] = []
            else:
                out[cur].append([float(t) for t in line.split()])
    return out


@pytest.fixture(scope="session")
def golden_five_points():
    return load_golden("five_points.txt")
