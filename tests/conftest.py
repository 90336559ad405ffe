import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden_path(name):
    return os.path.join(ROOT, "tests", "golden", name)


def read_golden_sections(name):
    """Parse a golden text file: '#' comments, '[section]' headers, rows of tokens."""
    sections, cur = {}, None
    with open(golden_path(name)) as fh:
        for raw in fh:
            line = raw.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                sections[cur] = []
            else:
                sections[cur].append(line.split())
    return sections


@pytest.fixture(scope="session")
def golden():
    return read_golden_sections
