import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse tests/golden/<name>: '#' comments, 'key = v1 v2 ...' integer/float lists."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            vals = [float(x) if ("." in x or "e" in x) else int(x) for x in v.split()]
            out[k.strip()] = vals
    return out


@pytest.fixture(scope="session")
def golden():
    return load_golden
