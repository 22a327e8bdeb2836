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


def live(msg):
    """A progress line that reaches the terminal while the test is still running (pytest holds back what a test prints
    until it ends; a test of several minutes would look dead meanwhile)."""
    capman = _CONFIG.pluginmanager.getplugin("capturemanager") if _CONFIG is not None else None
    if capman is None:
        print(msg, flush=True)
        return
    with capman.global_and_fixture_disabled():
        print(msg, flush=True)


def pytest_sessionstart(session):
    """The native libraries are loaded as built; only when none is there at all (a fresh checkout) are they built here."""
    from paper_2602_00328_amd import _build
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library(verbose=False)


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
