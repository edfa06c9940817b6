import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # load what is built; build only when nothing is
    from paper_2604_26557_amd import build
    build.build_if_missing()


def golden(name):
    """Parse tests/golden/<name>: 'key = value  # citation' lines into {key: int}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=")
            out[k.strip()] = int(v.strip().replace(",", "").replace("_", ""))
    return out


@pytest.fixture(scope="session")
def paper_sizes():
    return golden("paper_sizes.txt")
