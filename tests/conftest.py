import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def progress(msg: str) -> None:
    """Progress line for long GPU-box tests: written where the runner's watchdog sees it."""
    d = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(d):
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(msg + "\n")
    sys.stderr.write(msg + "\n")
    sys.stderr.flush()
