import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a `key: v0 v1 ...` fixture; `#` lines are the hand derivation."""
    rec = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val = line.split(":", 1)
            toks = val.split()
            rec[key.strip()] = toks[0] if key.strip() == "mode" else [int(t) for t in toks]
    return rec


def golden_files():
    """The single-row fixtures (w*.txt); a*.txt are fused-block fixtures."""
    return sorted(f for f in os.listdir(GOLDEN) if f.endswith(".txt") and f.startswith("w"))


@pytest.fixture(scope="session")
def oracle():
    import oracle as _o
    _o.load()
    return _o
