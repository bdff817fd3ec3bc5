import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, when no device is present and they were not asked for.
    try:
        import torch
        have = torch.cuda.is_available()
    except Exception:
        have = False
    if have:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(autouse=True)
def _tuning_overrides_follow_the_environment(monkeypatch):
    """The library reads its tuning overrides from the environment once; tests that set one through
    monkeypatch call `brg.brg_tuning_reload()` themselves, and this fixture reads the restored environment
    again after every test so that no override leaks into the next one."""
    yield
    monkeypatch.undo()
    try:
        import paper_1906_06440_amd as brg
        import os
        if os.path.exists(brg.lib_path()):
            brg.brg_tuning_reload()
    except Exception:
        pass
