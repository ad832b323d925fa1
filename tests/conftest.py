import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' comments, 'key values...' lines,
    'iter N' opens a new iteration record."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {"iters": []}
    cur = out
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "iter":
            cur = {}
            out["iters"].append(cur)
        elif key in ("hyper", "rule_c", "rule_a"):
            out[key] = {k: float(x) for k, x in (v.split("=") for v in vals)}
        elif key == "tensors":
            out["tensors"] = [int(x) for x in vals]
        else:
            cur[key] = [float(x) for x in vals]
    return out


@pytest.fixture(scope="session")
def golden_w2():
    return load_golden("hand_expanded_w2.txt")


@pytest.fixture(scope="session")
def golden_dcasgd():
    return load_golden("hand_expanded_dcasgd.txt")
