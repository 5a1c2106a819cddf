import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_available():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


class _ThkEnv:
    """Sets or removes THK_* environment switches for one test and makes the library read them
    (it reads them once per process, so a change needs thk_reload_env)."""

    def __init__(self, monkeypatch):
        self._mp = monkeypatch

    def setenv(self, name, value):
        import paper_2407_21018_amd as thk
        self._mp.setenv(name, value)
        thk.thk_reload_env()

    def delenv(self, name, raising=True):
        import paper_2407_21018_amd as thk
        self._mp.delenv(name, raising=raising)
        thk.thk_reload_env()


@pytest.fixture(autouse=True)
def _thk_env_restored():
    """Set up before any other fixture of a test, hence torn down last: after monkeypatch has put
    the environment back, the library re-reads its switches, so no test leaks its settings."""
    yield
    try:
        import paper_2407_21018_amd as thk
        thk.thk_reload_env()
    except ImportError:
        pass


@pytest.fixture
def thk_env(monkeypatch):
    return _ThkEnv(monkeypatch)


@pytest.fixture(params=["solo", "classic"])
def prune_launch(request, thk_env):
    """Both launch forms of thk_prune where the rows are held on chip: everything in one kernel
    (prologue block per unit, finisher), or state / main / repair kernels."""
    thk_env.setenv("THK_PRUNE_LAUNCH", request.param)
    return request.param


@pytest.fixture(params=["kernel", "fused"])
def decode_merge(request, thk_env):
    """Both ways of merging the split records of a decode call with at most 16 pieces: a second
    launch, or the last block of every head group inside the one launch."""
    thk_env.setenv("THK_DECODE_MERGE", request.param)
    return request.param
