import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")
    # Before anything touches a GPU: a library that is missing or was built from other sources than the
    # present ones is rebuilt here, so no test ever runs against a stale binary.
    from paper_2305_19982_amd import build

    if build.stale():
        build.build_libadama()


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped (not failed) where no device is visible, so a plain
    # `pytest tests/` on a CPU-only machine stays green.
    gpu_items = [it for it in items if "gpu" in it.keywords]
    if not gpu_items:
        return
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in gpu_items:
        it.add_marker(skip)
