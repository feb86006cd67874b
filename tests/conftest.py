import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: '# comment' lines and 'key: v v v' lines."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":", 1)
            nums = [float(v) for v in vals.split()]
            out[key.strip()] = nums[0] if len(nums) == 1 else nums
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden


@pytest.fixture
def progress(capsys):
    """Progress lines that reach the terminal while the test runs (past pytest's capture): a long test that stays
    silent for minutes looks hung to whoever watches the run."""
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return say
