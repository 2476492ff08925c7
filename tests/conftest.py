import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ppo():
    """The CPU oracle, compiled on first use."""
    from oracle import ppo as mod
    mod.build()
    return mod


def read_golden(name):
    """Parse a golden text fixture: '#' comments, 'key: ints...' lines -> dict of int lists."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, _, rest = line.partition(":")
            out.setdefault(key.strip(), []).append([int(x) for x in rest.split()])
    return out
