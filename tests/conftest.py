import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")
    import progress
    progress.capture_manager = config.pluginmanager.getplugin("capturemanager")


def load_golden(name):
    """Parse a 'key v v v' text fixture from tests/golden into {key: [ints]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = [int(x) for x in v]
    return out


@pytest.fixture(scope="session")
def example_A():
    g = load_golden("example_matrix_A.txt")
    return g
