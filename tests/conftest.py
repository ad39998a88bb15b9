import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_paper_pins():
    """tests/golden/paper_pins.txt -> {key: value string}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", "paper_pins.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, value, _cite = [p.strip() for p in line.split("|", 2)]
            out[key] = value
    return out


@pytest.fixture(scope="session")
def paper_pins():
    return load_paper_pins()
