import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name="paper_figures.txt"):
    vals = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.split("|")[0].strip()
            if not line or line.startswith("#"):
                continue
            key, val = [s.strip() for s in line.split("=")]
            vals[key] = float(val)
    return vals


@pytest.fixture(scope="session")
def golden():
    return load_golden()
