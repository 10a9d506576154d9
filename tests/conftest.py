import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


def _gpu_present() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        # the GPU cases name themselves (configuration, seed, shape) as they start, straight to
        # the terminal: a run that dies in a kernel still says which case it was in
        sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
        import gpu_util
        gpu_util.set_capture_manager(config.pluginmanager.get_plugin("capturemanager"))
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
