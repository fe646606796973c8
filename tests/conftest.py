import os
import sys
import time

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C-ABI library)")


def _progress(line: str) -> None:
    """Tests report their own progress into a log file (directory: $FIRP_TEST_LOG_DIR, else the
    scratch output folder at the repository root) so that a long, quiet GPU test is
    distinguishable from a hung one."""
    d = os.environ.get("FIRP_TEST_LOG_DIR") or os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "pytest_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {line}\n")
    except OSError:
        pass


@pytest.fixture
def progress():
    return _progress


def pytest_runtest_logstart(nodeid, location):
    _progress(f"start {nodeid}")


def pytest_runtest_logfinish(nodeid, location):
    _progress(f"done  {nodeid}")
