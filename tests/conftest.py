import os
import sys

import pytest

# The GPU tests run the copy-engine path the way the package sets a process up (stream
# waits carried out by the command processor); the variable must be there before the
# HIP runtime starts, so it is set before anything imports torch.
os.environ.setdefault("GPU_STREAMOPS_CP_WAIT", "1")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
