import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped where no GPU is visible, so a plain `pytest tests/` is green on a CPU machine."""
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


class _SwitchEnv:
    """pytest's monkeypatch with one addition: after every change of the environment the library re-reads its
    DCHAG_* debugging switches (it reads them once, when it is loaded, and never during a call)."""

    def __init__(self, mp):
        self._mp = mp

    @staticmethod
    def _reload():
        import paper_2506_21411_amd as dchag
        if os.path.exists(dchag.library_path()):
            dchag.dchag_debug_reload()

    def setenv(self, *a, **k):
        self._mp.setenv(*a, **k)
        self._reload()

    def delenv(self, *a, **k):
        self._mp.delenv(*a, **k)
        self._reload()

    def __getattr__(self, name):
        return getattr(self._mp, name)


@pytest.fixture
def monkeypatch(monkeypatch):
    proxy = _SwitchEnv(monkeypatch)
    yield proxy
    monkeypatch.undo()
    proxy._reload()
