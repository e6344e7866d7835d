import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no GPU is visible.
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


def set_flags(monkeypatch, add: str = "", remove: str = "") -> None:
    """For the rest of the test, every call through the binding passes the hstu_flags named in
    `add` as well (e.g. "NO_PACK"), and no longer the one named in `remove`."""
    from paper_2508_04711_amd import binding

    def bit(name):
        return getattr(binding, "HSTU_FLAG_" + name) if name else 0
    monkeypatch.setattr(binding, "default_flags", (binding.default_flags | bit(add)) & ~bit(remove))
