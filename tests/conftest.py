import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")


def read_golden_values(name):
    """Parse tests/golden/<name>: 'key = v v v' lines, '#' comments; ints decimal or 0x-hex."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if "=" in line:
                k, v = line.split("=", 1)
                out[k.strip()] = [int(t, 0) for t in v.split()]
            else:
                out.setdefault("_list", []).append(int(line, 0))
    return out


@pytest.fixture(scope="session")
def worked():
    return read_golden_values("worked_values.txt")
