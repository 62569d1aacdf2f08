import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C-ABI)")


def parse_fixture(path):
    """Plain-text fixture: '#' comments, 'key: v v v' lines -> dict of key -> list of floats/ints."""
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            out.setdefault(key.strip(), []).append([float(v) if "." in v else int(v) for v in vals.split()])
    return out


GOLDEN = os.path.join(ROOT, "tests", "golden")
