import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

_CONFIG = None


def pytest_configure(config):
    global _CONFIG
    _CONFIG = config
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def progress(msg: str) -> None:
    """Print a line past pytest's output capture (long GPU tests must show signs of life)."""
    capman = _CONFIG.pluginmanager.getplugin("capturemanager") if _CONFIG is not None else None
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print(msg, file=sys.stderr, flush=True)
    else:
        print(msg, file=sys.stderr, flush=True)
