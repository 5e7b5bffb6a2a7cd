import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs the HIP library through its C ABI)")
    config.addinivalue_line("markers", "slow: CPU test of many minutes; runs only with BCS_RUN_SLOW=1 in the environment")


def pytest_collection_modifyitems(config, items):
    if os.environ.get("BCS_RUN_SLOW") == "1":
        return
    skip = pytest.mark.skip(reason="slow: set BCS_RUN_SLOW=1 to run")
    for item in items:
        if "slow" in item.keywords:
            item.add_marker(skip)


def load_table(name):
    """Parse a tests/golden table: returns (p, q, baseblocks, recv[p][q], send[p][q])."""
    import numpy as np
    rows = []
    p = q = None
    with open(os.path.join(GOLDEN, name + ".txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("p "):
                tok = line.split()
                p, q = int(tok[1]), int(tok[3])
                continue
            rows.append([int(v) for v in line.split()])
    a = np.array(rows, dtype=np.int32)
    assert a.shape == (2 + 2 * q, p)
    assert (a[0] == np.arange(p)).all()
    return p, q, a[1], a[2:2 + q].T.copy(), a[2 + q:].T.copy()


@pytest.fixture(scope="session")
def oracle():
    import oracle as orc
    orc.build(force=False)
    return orc
