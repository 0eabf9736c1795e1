import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU harness)")


def golden_lines(name):
    """Non-comment, non-empty lines of a fixture under tests/golden/."""
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.rstrip("\n") for ln in f if ln.strip() and not ln.lstrip().startswith("#")]


@pytest.fixture(scope="session")
def table2():
    """Table II as a list of (case, modesA, modesB, [kernel strings])."""
    rows = []
    for ln in golden_lines("table2_cases.txt"):
        f = [x.strip() for x in ln.split("|")]
        rows.append((f[0], f[1], f[2], [k for k in f[3:] if k]))
    return rows
