"""Algorithmic bytes of one decode step: what the method itself must read from HBM.

Per token with exit position e and T attended positions:
    bytes(e, T) = e * W16 + (L - e) * W4 + H + L * kv * T
W16: a backbone block (seven matrices + two norm gains) in the storage dtype;
W4:  its river twin (4-bit codes + scale and zero per group + the same norm gains);
H:   final norm + LM head + one embedding row;  kv: K and V of one position of one block.
Writes (one K/V row per block, a few activation vectors) are negligible and not counted.
Host arithmetic on shapes only.
"""
from __future__ import annotations

from .configs import MATRICES, ModelConfig, matrix_shape


def elem_bytes(cfg: ModelConfig) -> int:
    return 2 if cfg.dtype == 1 else 4


def block_bytes_backbone(cfg: ModelConfig) -> int:
    return (cfg.params_per_block + 2 * cfg.d_model) * elem_bytes(cfg)


def block_bytes_river(cfg: ModelConfig) -> int:
    es = elem_bytes(cfg)
    total = 2 * cfg.d_model * es
    for m in MATRICES:
        rows, cols = matrix_shape(cfg, m)
        groups = -(-cols // cfg.river_group)
        total += rows * cols // 2 + 2 * rows * groups * es
    return total


def head_bytes(cfg: ModelConfig) -> int:
    return (cfg.vocab * cfg.d_model + 2 * cfg.d_model) * elem_bytes(cfg)


def kv_bytes_per_position(cfg: ModelConfig) -> int:
    """K and V of one cached position, summed over all blocks."""
    return 2 * cfg.n_kv_heads * cfg.head_dim * elem_bytes(cfg) * cfg.n_layers


def step_bytes(cfg: ModelConfig, exit_pos: int, attended: int) -> int:
    e = exit_pos
    return (e * block_bytes_backbone(cfg) + (cfg.n_layers - e) * block_bytes_river(cfg)
            + head_bytes(cfg) + kv_bytes_per_position(cfg) * attended)


def backbone_param_bytes(cfg: ModelConfig) -> int:
    """All backbone parameters (embedding and LM head untied)."""
    es = elem_bytes(cfg)
    return (cfg.n_layers * (cfg.params_per_block + 2 * cfg.d_model)
            + 2 * cfg.vocab * cfg.d_model + cfg.d_model) * es


def kv_cache_bytes(cfg: ModelConfig, context: int) -> int:
    return kv_bytes_per_position(cfg) * context


def batch_step_bytes(cfg: ModelConfig, exit_positions, attended) -> int:
    """One batched decode step: block l (1-based) reads the backbone matrices if any sequence
    is still in the backbone there (exit position >= l) and the river twin if any sequence has
    left it (exit position < l); the head once; every sequence its own K/V."""
    total = head_bytes(cfg)
    for l in range(1, cfg.n_layers + 1):
        if any(e >= l for e in exit_positions):
            total += block_bytes_backbone(cfg)
        if any(e < l for e in exit_positions):
            total += block_bytes_river(cfg)
    total += sum(kv_bytes_per_position(cfg) * t for t in attended)
    return total
