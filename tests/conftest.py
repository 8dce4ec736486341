import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden_kv(name):
    """Parse a 'key value unit  # comment' fixture into {key: float}."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                parts = line.split()
                out[parts[0]] = float(parts[1])
    return out


def read_golden_ring_example(name):
    """Parse a 'dims / inputs / expected' fixture."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                parts = line.split()
                out[parts[0]] = [float(x) for x in parts[1:]]
    out["dims"] = [int(x) for x in out["dims"]]
    return out
