import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse tests/golden/<name>: '#' comments, 'key: v v v' lines, ';' rows."""
    out = {}
    path = os.path.join(ROOT, "tests", "golden", name)
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val = line.split(":", 1)
            rows = [[float(x) if ("." in x or "e" in x) else int(x)
                     for x in r.split()] for r in val.split(";")]
            out[key.strip()] = rows if len(rows) > 1 else rows[0]
    return out


@pytest.fixture(scope="session")
def golden():
    return load_golden
