"""The byte model (roofline denominator) against the closed forms the paper prints."""
import os

import pytest

from paper_2604_18396_amd import byte_model as bm
from paper_2604_18396_amd import configs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_memory_table_backbone.txt")


def test_backbone_rows_of_the_paper_memory_table():
    cfg = configs.LLAMA_8B
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for ctx, params_gb, kv_mb in rows:
        assert bm.backbone_param_bytes(cfg) / 2 ** 30 == pytest.approx(float(params_gb), abs=0.005)
        assert bm.kv_cache_bytes(cfg, int(ctx)) / 2 ** 20 == float(kv_mb)


def test_step_bytes_decomposition():
    cfg = configs.LLAMA_8B
    w16, w4, h = bm.block_bytes_backbone(cfg), bm.block_bytes_river(cfg), bm.head_bytes(cfg)
    assert w16 == 2 * 218_103_808 + 4 * 4096
    # 4.5 bits per weight with group 64 and bf16 scale/zero
    assert w4 == 218_103_808 * 9 // 16 + 4 * 4096
    assert 0.28 < w4 / w16 < 0.2815
    assert bm.kv_bytes_per_position(cfg) == 128 * 1024
    L = cfg.n_layers
    assert bm.step_bytes(cfg, L, 512) == L * w16 + h + 512 * 128 * 1024
    assert bm.step_bytes(cfg, 18, 512) - bm.step_bytes(cfg, 17, 512) == w16 - w4
    # the whole dense step reads every backbone parameter but the embedding table once
    assert bm.step_bytes(cfg, L, 0) == bm.backbone_param_bytes(cfg) - (cfg.vocab - 1) * cfg.d_model * 2
    # ragged last group (C1's 688-column down projection has 11 groups per row)
    t = configs.TINY
    assert bm.block_bytes_river(t) > t.params_per_block // 2


def test_batch_step_bytes_reduces_to_the_single_sequence_model():
    from paper_2604_18396_amd import byte_model, configs
    cfg = configs.LLAMA_8B
    for e in (8, 18, 32):
        assert byte_model.batch_step_bytes(cfg, [e], [700]) == byte_model.step_bytes(cfg, e, 700)
    # two sequences at depths 10 and 20: blocks 1..10 backbone only, 11..20 both sets, 21..32 river only
    b = byte_model.batch_step_bytes(cfg, [10, 20], [100, 200])
    want = (20 * byte_model.block_bytes_backbone(cfg) + 22 * byte_model.block_bytes_river(cfg)
            + byte_model.head_bytes(cfg) + byte_model.kv_bytes_per_position(cfg) * 300)
    assert b == want
