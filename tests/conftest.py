import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


CAPTURE_MANAGER = None


def pytest_configure(config):
    global CAPTURE_MANAGER
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    CAPTURE_MANAGER = config.pluginmanager.getplugin("capturemanager")


def progress(msg: str) -> None:
    """Print a progress line past pytest's output capture (long GPU runs must show signs of life)."""
    if CAPTURE_MANAGER is not None:
        with CAPTURE_MANAGER.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)


@pytest.fixture(scope="session")
def repo_root():
    return ROOT
