import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def micro_shape():
    """A model small enough for exhaustive checks of the oracle."""
    from synth import HawkShape
    return HawkShape("micro", n_layers=2, d_model=32, n_heads=4, d_mlp=48, vocab=40,
                     n_cond=5, grid_h=4, grid_w=4, k=3, dtype="fp32", top_k=40)
