import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_setup():
    """C1 shape: weights, oracle river tensors (all on the CPU)."""
    from oracle import river_oracle as ro
    from paper_2604_18396_amd import configs, inputs
    cfg = configs.TINY
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    river = ro.quantize_river(cfg, w)
    return cfg, w, river
