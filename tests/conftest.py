import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests use the library that is built; they build it only if none is there.
    from paper_2512_22142_amd.build import ensure_built
    ensure_built()


def read_golden(name):
    """Parses a `key value...` text fixture under tests/golden/ (lines starting
    with # are citations / comments)."""
    rows = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            parts = line.split()
            rows[parts[0]] = parts[1:]
    return rows


@pytest.fixture(scope="session")
def golden():
    return read_golden
