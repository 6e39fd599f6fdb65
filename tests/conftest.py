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
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def nsk_env(monkeypatch):
    """Sets one of libnsk's NSK_* test switches for the duration of a test.  The library reads its switches once,
    so every change (and the restoration afterwards) is followed by nsk_test_hooks_reload()."""
    from paper_2409_11600_amd import binding

    def set_switch(name, value):
        monkeypatch.setenv(name, value)
        binding.lib().nsk_test_hooks_reload()

    yield set_switch
    monkeypatch.undo()
    binding.lib().nsk_test_hooks_reload()
