import os
import sys
import time

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C-ABI library)")


def _log_dir():
    """Where tests report their own progress: $FIRP_TEST_LOG_DIR if set; otherwise, on a machine
    with a GPU only, the scratch output folder at the repository root (a long, quiet GPU test
    must be distinguishable from a hung one); CPU-only runs write nothing."""
    d = os.environ.get("FIRP_TEST_LOG_DIR")
    if d:
        return d
    global _HAS_GPU
    if _HAS_GPU is None:
        try:
            import torch
            _HAS_GPU = bool(torch.cuda.is_available())
        except Exception:
            _HAS_GPU = False
    return os.path.join(ROOT, "gpurun_out") if _HAS_GPU else None


_HAS_GPU = None


def _progress(line: str) -> None:
    d = _log_dir()
    if not d:
        return
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
