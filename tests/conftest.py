import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no GPU is visible (they are selected with -m gpu on the GPU machine)
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session")
def tiny():
    """Tiny head (d=256, 4x64 query heads, 2 KV heads, ffn 688, vocab 4096): weights, inputs, subset."""
    from paper_2509_18362_amd import synth
    wl = synth.WORKLOADS["c1_tiny"]
    w = synth.make_weights(wl)
    act = synth.make_activations(wl)
    ids = synth.make_subsets(wl)[0]
    return {"wl": wl, "shape": wl.shape, "w": w, "act": act, "ids": ids}
