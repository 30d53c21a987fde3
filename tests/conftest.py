import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Read a fixture: '#' comment lines (the citation), then one JSON document."""
    with open(os.path.join(GOLDEN, name)) as f:
        body = "".join(line for line in f if not line.lstrip().startswith("#"))
    return json.loads(body)


@pytest.fixture(scope="session")
def golden():
    return load_golden
