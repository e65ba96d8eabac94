import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# test_oracle_mutants.py points this at a directory holding a deliberately broken copy of
# oracle/ and expects the pins to fail; nothing else sets it.
if os.environ.get("TIDE_ORACLE_PARENT"):
    sys.path.insert(0, os.environ["TIDE_ORACLE_PARENT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


def read_golden(path):
    """Parse a 'key: v1 v2 ...' text fixture; lines starting with # are citations."""
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            out[key.strip()] = val.split()
    return out
