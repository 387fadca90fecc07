import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on a GPU box)")


def load_golden(name):
    """Parse tests/golden/<name>: {case: {key: [floats]}}."""
    cases, cur = {}, None
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("case "):
                cur = cases.setdefault(line[5:].strip(), {})
            else:
                key, vals = line.split(":", 1)
                cur[key.strip()] = [float(v) for v in vals.split()]
    return cases


@pytest.fixture(scope="session")
def golden():
    return load_golden("hand_examples.txt")
