import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# The tests with several best-effort clients need 2 + 2n hardware queues; HIP reads the
# variable when it initialises, so it is set here, before any test imports torch.
# (an inherited smaller value, such as a machine-wide default of 4, is raised)
try:
    _have = int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))
except ValueError:
    _have = 4
if _have < 20:
    os.environ["GPU_MAX_HW_QUEUES"] = "20"


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
