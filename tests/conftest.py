import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def torch_mod():
    """torch with a visible GPU and the HIP library loaded (no fallback: a missing library is an error)."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2510_03283_amd import binding
    binding.load()
    return torch


@pytest.fixture(scope="session")
def weights_7b():
    """Weights of the 7B-class layer, drawn once per test session (seed of the `7b` configuration)."""
    from paper_2510_03283_amd import synth
    return synth.make_weights(synth.CONFIGS["7b"])
