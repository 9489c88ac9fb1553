import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture
def sol_env(monkeypatch):
    """Set a tuning override of the library for one test: the library reads its environment overrides once,
    so it is told to read them again after every change and after the test."""
    from paper_2205_10357_amd import binding as B

    def set_override(name, value):
        monkeypatch.setenv(name, str(value))
        B.sol_reload_overrides()

    yield set_override
    monkeypatch.undo()
    B.sol_reload_overrides()
