import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture into {key: [token lists]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            out.setdefault(tok[0], []).append(tok[1:])
    return out


@pytest.fixture(scope="session")
def worked_example():
    g = load_golden("wros_worked_example.txt")
    val = dict(zip(g["letters"][0], (float(v) for v in g["standins"][0])))
    return g, val
