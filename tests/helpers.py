"""Helpers shared by the test files (input construction only; no expected values)."""
import numpy as np
import torch

# uses of the near-tie rule for greedy tokens in the GPU parity tests (see check_token there)
NEAR_TIES: list = []


def grid_weights(rows, cols, group, dtype, seed):
    """Weights that already lie on a 4-bit grid: w = (q - z) * 2^-k with integer z, every
    group containing the codes 0 and 15, so the quantiser must give them back exactly."""
    rng = np.random.default_rng(seed)
    w = np.empty((rows, cols), dtype=np.float64)
    for c0 in range(0, cols, group):
        n = min(group, cols - c0)
        q = rng.integers(0, 16, size=(rows, n))
        q[:, 0], q[:, 1] = 0, 15
        q = rng.permuted(q, axis=1)
        z = rng.integers(1, 15, size=(rows, 1))
        k = rng.integers(5, 9, size=(rows, 1))
        w[:, c0:c0 + n] = (q - z) * 2.0 ** (-k)
    return torch.from_numpy(w).to(dtype)


def grid_model(cfg, seed):
    """A full weight set whose seven block matrices all lie on the 4-bit grid of the river
    format; embedding and head are ordinary random matrices."""
    from paper_2604_18396_amd import inputs
    from paper_2604_18396_amd.configs import MATRICES, matrix_shape
    tdt = torch.bfloat16 if cfg.dtype == 1 else torch.float32
    w = inputs.make_weights(cfg, seed)
    for l, blk in enumerate(w["layers"]):
        for m, name in enumerate(MATRICES):
            rows, cols = matrix_shape(cfg, name)
            # scale the grid down so activations stay in a sane range
            blk[name] = (grid_weights(rows, cols, cfg.river_group, torch.float64,
                                      seed * 1000 + l * 10 + m) / 16.0).to(tdt)
    return w
