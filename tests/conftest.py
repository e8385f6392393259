import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture into {section: list of rows of tokens}."""
    out, cur = {}, None
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                out[cur] = []
            else:
                out[cur].append(line.split())
    return out


@pytest.fixture(scope="session")
def golden_fig2():
    return read_golden("fig2_worked_example.txt")
