import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _automatic_decode_kernel_choice_after_every_test():
    """Tests that force the generic decode kernel must not leak the switch into later tests."""
    yield
    mod = sys.modules.get("paper_2605_19660_amd.binding")
    if mod is not None and getattr(mod, "_lib", None) is not None:
        mod.debug_force_generic_decode(False)
