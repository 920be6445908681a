import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an AMD GPU (run with -m gpu on the MI355X box)")


def load_golden(name):
    """Parse a tests/golden text fixture: '#' comments and 'name = python-literal' lines."""
    import ast
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition("=")
            out[key.strip()] = ast.literal_eval(val.strip())
    return out


@pytest.fixture(scope="session")
def golden():
    return load_golden
