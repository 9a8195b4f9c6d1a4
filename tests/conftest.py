import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' comments, then 'key value' lines."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                key, val = line.split(None, 1)
                out[key] = val.strip()
    return out


@pytest.fixture(scope="session")
def paper_hp():
    g = read_golden("hyperparameters.txt")
    return {k: float(v) for k, v in g.items()}
