import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def tiny_cfg():
    from synth import ModelConfig
    # a small model that still has >1 layer, several heads, partial rotary and a ragged head_dim
    return ModelConfig(n_layers=2, d_model=48, n_heads=3, head_dim=16, rotary_dims=4, d_ff=96,
                       vocab=160, dtype="fp32", pad_id=150)
