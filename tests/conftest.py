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
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


# ---- shared by the full-size GPU parity tests (configs 2, 3 and 4 use the same Mixtral-shaped layer)
@pytest.fixture(scope="session")
def mixtral_layer():
    """(cfg, (Wg, b, experts)) of benchmark config 2: layer 0 of the synthetic Mixtral-shaped stack."""
    from paper_2512_03927_amd import synth
    cfg = synth.CONFIGS[2]
    return cfg, synth.layer_weights(cfg, 0)


@pytest.fixture(scope="session")
def mixtral_experts_f64(mixtral_layer):
    """The eight experts widened once to float64 (W1, W3, W2) tuples for the oracle: widening the
    stored bf16 is nearly all of the oracle's time per token, so with this it checks every token
    of the full-size configurations instead of a sample (22.5 GB of host memory)."""
    from oracle import moe_oracle as O
    cfg, (_, _, experts) = mixtral_layer
    return [tuple(O.widen(w) for w in O.split_expert(e, cfg.hidden, cfg.ffn)) for e in experts]
