"""Pins for the oracle's 4-bit river format ("KV-Shared Exit Layer": W4A16 weight-only PTQ).

The quantiser is pinned by the properties the definition fixes (range, error bound,
exact round trip on grid weights, constant groups) and by a second, independent
statement of the same definition in numpy/torch (oracle/plain_definition.py)."""
import numpy as np
import pytest
import torch

from oracle import plain_definition as pd
from oracle import river_oracle as ro
from helpers import grid_weights


def _rand(rows, cols, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(rows, cols, generator=g) * 0.02).to(dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("cols,group", [(256, 64), (688, 64), (128, 32)])
def test_codes_range_and_error_bound(dtype, cols, group):
    w = _rand(48, cols, dtype, 3)
    codes, scale, zero = ro.quantize_w4(w, group)
    assert codes.dtype == torch.uint8 and codes.shape == (48, cols // 2)
    gpr = -(-cols // group)
    assert scale.shape == (48, gpr) and zero.shape == (48, gpr)
    deq = ro.dequantize_w4(codes, scale, zero, group)
    s = scale.double().repeat_interleave(group, dim=1)[:, :cols].numpy()
    z = zero.double().repeat_interleave(group, dim=1)[:, :cols].numpy()
    err = np.abs(deq - w.double().numpy())
    # round-to-nearest on the grid: half a step, plus what storing scale/zero in the
    # weight dtype can move the grid end points (zero has |z| <= ~16, scale is one step)
    ulp = 2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -24
    slack = s * (np.abs(z) + 16) * ulp
    assert np.all(err <= 0.5 * s + slack + 1e-12)
    assert np.all(s > 0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_two_statements_of_the_format_agree(dtype):
    for cols, group, seed in [(256, 64, 1), (688, 64, 2), (64, 16, 3)]:
        w = _rand(40, cols, dtype, seed)
        a = ro.quantize_w4(w, group)
        b = pd.quantize_w4(w, group)
        for x, y in zip(a, b):
            assert torch.equal(x, y)
        np.testing.assert_array_equal(ro.dequantize_w4(*a, group), pd.dequantize_w4(*b, group))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_grid_round_trip_exact(dtype):
    w = grid_weights(32, 688, 64, dtype, 11)
    assert torch.equal(w.double(), grid_weights(32, 688, 64, torch.float64, 11))  # representable
    codes, scale, zero = ro.quantize_w4(w, 64)
    np.testing.assert_array_equal(ro.dequantize_w4(codes, scale, zero, 64), w.double().numpy())
    # scale is the power of two and zero the integer the weights were built from
    assert torch.all(torch.log2(scale.double()) == torch.log2(scale.double()).round())
    assert torch.all(zero.double() == zero.double().round())


def test_constant_group():
    w = torch.full((4, 128), 0.0123, dtype=torch.float32)
    w[1] = -2.5
    w[2] = 0.0
    codes, scale, zero = ro.quantize_w4(w, 64)
    assert torch.all(scale == 1.0)
    assert torch.all(codes == 0)
    np.testing.assert_array_equal(ro.dequantize_w4(codes, scale, zero, 64), w.double().numpy())


def test_extremes_hit_codes_0_and_15_and_nibble_order():
    w = torch.linspace(-1.0, 1.0, 64, dtype=torch.float32)[None, :].contiguous()
    codes, scale, zero = ro.quantize_w4(w, 64)
    q = torch.stack([codes & 15, codes >> 4], dim=2).reshape(1, 64)   # even index = low nibble
    assert q[0, 0] == 0 and q[0, -1] == 15
    assert torch.all(q[0, 1:] >= q[0, :-1])                           # monotone input, monotone codes
    assert scale[0, 0].item() == pytest.approx(2.0 / 15.0, rel=1e-6)
    assert zero[0, 0].item() == pytest.approx(7.5, rel=1e-6)
