import os
import sys

import pytest

# the kernel-shape overrides the GPU tests use (DG_ONEHOT_PLAN, ...) are honoured only under this guard, which the
# library reads once, at its first call
os.environ["DG_TEST_OVERRIDES"] = "1"

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
