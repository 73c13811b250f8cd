import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")

# The library reads its COMMFUSE_* tuning overrides once, at its first call; the tests switch them between
# calls (to force every tile shape and code path), so they ask for the environment to be read on every call.
os.environ.setdefault("COMMFUSE_TUNING_LIVE", "1")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return GOLDEN
