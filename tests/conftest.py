import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_paper_numbers():
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", "paper_numbers.txt")) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if line:
                key, val = line.split()
                out[key] = float(val)
    return out


@pytest.fixture(scope="session")
def paper_numbers():
    return load_paper_numbers()
