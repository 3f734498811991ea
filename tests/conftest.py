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
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session")
def experts_8x22b():
    """One set of Mixtral-8x22B-shaped expert weights shared by every 8x22B GPU case (their
    token and router seeds still differ per case): ((W1, W3, W2) on the GPU, their bf16 bits
    on the host)."""
    from paper_2605_17889_amd import synth
    cfg = synth.PRESETS["mixtral8x22b_prefill"]
    print("generating 8x22B-shaped expert weights on the GPU", flush=True)
    W1, W3, W2 = synth.make_experts(cfg, "cuda")
    host = tuple(synth.bf16_bits(w) for w in (W1, W3, W2))
    return (W1, W3, W2), host
