import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_table(name):
    """Parse a schedule table fixture: returns (p, b, recv[k][r], send[k][r])."""
    p, b, recv, send = None, None, {}, {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            vals = [int(v) for v in vals]
            if key == "p":
                p = vals[0]
            elif key == "b":
                b = vals
            elif key.startswith("recv"):
                recv[int(key[4:])] = vals
            elif key.startswith("send"):
                send[int(key[4:])] = vals
    q = len(recv)
    return p, b, [recv[k] for k in range(q)], [send[k] for k in range(q)]


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle._load()
    return oracle
