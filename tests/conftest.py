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


def pytest_terminal_summary(terminalreporter):
    """How often a GPU parity test accepted a greedy token that differs from the oracle's
    on a numerical near-tie of the two best logits (bf16 only; fp32 must match)."""
    try:
        import helpers
    except ImportError:
        return
    terminalreporter.write_line(f"near-tie token acceptances: {len(helpers.NEAR_TIES)}")
    for line in helpers.NEAR_TIES:
        terminalreporter.write_line("  " + line)
