import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: 'key v v v' lines, '#' comments; repeated keys accumulate."""
    out = {}
    for line in (ROOT / "tests" / "golden" / name).read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, _, rest = line.partition(" ")
        out.setdefault(key, []).append(rest.strip())
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
