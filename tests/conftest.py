import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu; when collected on a machine without a GPU they skip.
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this machine")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


class _Tune:
    """Sets the library's tuning overrides (tp_layer_set_option) for one test; all are cleared afterwards."""
    NAMES = ("gemm_tile", "gemm_shares", "gemm_band", "gemm_force", "attn_chunk", "fuse_colsum", "side_chains")

    def set(self, name, value):
        import paper_2111_05972_amd as pkg
        pkg.tp_layer_set_option(name, value)

    def clear(self):
        for n in self.NAMES:
            self.set(n, None)


@pytest.fixture
def tune():
    t = _Tune()
    t.clear()
    yield t
    t.clear()
