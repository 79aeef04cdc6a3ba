"""Seeded synthetic inputs: weights, prompts, exit schedules.

This module is the only code shared by the HIP path's tests/bench and the CPU
oracle.  It draws random numbers and nothing else: no normalisation, rotation,
attention, quantisation or similarity arithmetic lives here.

Weights are i.i.d. N(0, 0.02^2) (norm gains are 1), stored as torch CPU tensors
in the model's dtype; prompts are uniform token ids; forced exit schedules
follow a two-component uniform mixture with about half of the tokens leaving
the backbone in its first half.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from .configs import DTYPE_BF16, MATRICES, ModelConfig, matrix_shape

_CHUNK_ELEMS = 1 << 22
_STD = 0.02


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _fill_normal(out: np.ndarray, seed_key: tuple[int, ...]) -> None:
    """Fill a 2-D float32 array with N(0, _STD^2).

    The array is cut into fixed row chunks, each with its own generator keyed
    by (seed_key, chunk), so the values do not depend on the thread count.
    """
    rows, cols = out.shape
    rpc = max(1, _CHUNK_ELEMS // cols)
    jobs = [(c, r0, min(rows, r0 + rpc)) for c, r0 in enumerate(range(0, rows, rpc))]

    def run(job):
        c, r0, r1 = job
        rng = np.random.default_rng(list(seed_key) + [c])
        rng.standard_normal(out=out[r0:r1], dtype=np.float32)
        out[r0:r1] *= np.float32(_STD)

    if len(jobs) == 1:
        run(jobs[0])
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(run, jobs))


def _normal_tensor(shape: tuple[int, int], seed_key: tuple[int, ...], dtype: int) -> torch.Tensor:
    a = np.empty(shape, dtype=np.float32)
    _fill_normal(a, seed_key)
    t = torch.from_numpy(a)
    if dtype == DTYPE_BF16:
        t = t.to(torch.bfloat16)      # round-to-nearest-even storage conversion
    return t.contiguous()


def _gain(n: int, seed_key: tuple[int, ...], std: float, tdt) -> torch.Tensor:
    """Norm gains: ones, or 1 + N(0, std^2) drawn from the generator keyed by seed_key."""
    if std <= 0.0:
        return torch.ones(n, dtype=tdt)
    g = 1.0 + std * np.random.default_rng(list(seed_key)).standard_normal(n).astype(np.float32)
    return torch.from_numpy(g).to(tdt).contiguous()


def make_weights(cfg: ModelConfig, seed: int, layers: range | None = None, gain_std: float = 0.0) -> dict:
    """Random-init backbone weights.

    Returns {"tok_emb", "final_norm", "lm_head", "layers": [ {attn_norm, wq, wk,
    wv, wo, ffn_norm, w_gate, w_up, w_down}, ... ]}; matrices are [out, in]
    row-major.  `layers` restricts generation to a sub-range (others are None).
    gain_std > 0 draws the norm gains as 1 + N(0, gain_std^2) instead of ones.
    """
    tdt = torch.bfloat16 if cfg.dtype == DTYPE_BF16 else torch.float32
    w = {
        "tok_emb": _normal_tensor((cfg.vocab, cfg.d_model), (seed, 0, 0), cfg.dtype),
        "lm_head": _normal_tensor((cfg.vocab, cfg.d_model), (seed, 0, 1), cfg.dtype),
        "final_norm": _gain(cfg.d_model, (seed, 0, 2), gain_std, tdt),
        "layers": [],
    }
    want = set(layers) if layers is not None else set(range(cfg.n_layers))
    for l in range(cfg.n_layers):
        if l not in want:
            w["layers"].append(None)
            continue
        blk = {"attn_norm": _gain(cfg.d_model, (seed, l + 1, 100), gain_std, tdt),
               "ffn_norm": _gain(cfg.d_model, (seed, l + 1, 101), gain_std, tdt)}
        for m, name in enumerate(MATRICES):
            blk[name] = _normal_tensor(matrix_shape(cfg, name), (seed, l + 1, m), cfg.dtype)
        w["layers"].append(blk)
    return w


def make_prompt(vocab: int, n: int, seed: int) -> np.ndarray:
    """n token ids ~ U{0..vocab-1}, int32."""
    return np.random.default_rng(seed).integers(0, vocab, size=n, dtype=np.int32)


def make_exit_schedule(n_layers: int, n: int, seed: int) -> np.ndarray:
    """n forced exit positions, int32.

    With probability 1/2 the position is uniform on {L/4 .. L/2}, otherwise
    uniform on {L/2+1 .. L-1}.  Two draws per step: the first picks the half.
    """
    rng = np.random.default_rng(seed)
    lo0, lo1 = n_layers // 4, n_layers // 2
    hi0, hi1 = n_layers // 2 + 1, n_layers - 1
    out = np.empty(n, dtype=np.int32)
    for i in range(n):
        first = rng.random() < 0.5
        out[i] = rng.integers(lo0, lo1 + 1) if first else rng.integers(hi0, hi1 + 1)
    return out
