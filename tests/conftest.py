import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the long GPU tests carry @pytest.mark.timeout(...): without the plugin the mark would silently do nothing
    if not config.pluginmanager.hasplugin("timeout"):
        config.addinivalue_line("markers", "timeout: per-test time limit (pytest-timeout is NOT installed: no limit is enforced)")
        import warnings
        warnings.warn("pytest-timeout is not installed: the time limits of the GPU tests are not enforced")


def pytest_collection_modifyitems(config, items):
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
