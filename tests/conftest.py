import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C ABI)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: `key: v0 v1 ...` lines, `#` comments."""
    out = {}
    path = os.path.join(ROOT, "tests", "golden", name)
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            out[key.strip()] = [float(eval(v, {"__builtins__": {}})) for v in vals.split()]
    return out
