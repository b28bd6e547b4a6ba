import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs the HIP library through its C ABI)")


def golden_lines(name, kind=None):
    """Non-comment lines of a golden text fixture, split into fields."""
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            fields = line.replace("->", " ").split()
            if kind is None or fields[0] == kind:
                rows.append(fields)
    return rows


@pytest.fixture(scope="session")
def oracle():
    import oracle as orc
    orc.lib()
    return orc
