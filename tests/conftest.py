import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: '[section]' headers followed by rows
    of integers; '#' lines are comments."""
    path = os.path.join(ROOT, "tests", "golden", name)
    sections, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                sections[cur] = []
            else:
                sections[cur].append([int(v) for v in line.split()])
    return {k: np.array(v) for k, v in sections.items()}


@pytest.fixture(scope="session")
def hand_example():
    return load_golden("hand_example_v4.txt")
