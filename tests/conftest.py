import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# A decode batch whose sequences all fit 14 blocks is planned without any sharing or cutting (it is bound by launch
# latency).  The tests exercise the sharing and split-K machinery at exactly such sizes, where the oracle is fast, so
# they switch that shortcut off; the tests of the shortcut itself switch it back on.
os.environ.setdefault("GLM_PLAN_TINY_BLOCKS", "0")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (run with -m gpu)")


def _has_gpu() -> bool:
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
