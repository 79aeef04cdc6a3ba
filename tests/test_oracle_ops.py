"""Pins for the oracle's building blocks: each is checked against a library routine,
a closed form or an invariant, never against a retyped copy of its own formula."""
import ctypes as C

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import river_oracle as ro

RNG = np.random.default_rng(7)


def _p(a):
    return a.ctypes.data


def rmsnorm(x, g, eps):
    out = np.empty_like(x)
    g32 = np.ascontiguousarray(g, dtype=np.float32)
    ro.lib().orc_rmsnorm(_p(x), _p(g32), 0, len(x), eps, _p(out))
    return out


def rope(v, n_heads, hd, pos, base):
    v = np.ascontiguousarray(v, dtype=np.float64).copy()
    ro.lib().orc_rope(_p(v), n_heads, hd, pos, base)
    return v


def attention(q, K, V, nq, nkv, hd):
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    o = np.empty(nq * hd)
    ro.lib().orc_attention(_p(q), _p(K), _p(V), K.shape[0], nq, nkv, hd, _p(o))
    return o


def cosine(a, b):
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    return ro.lib().orc_cosine(_p(a), _p(b), len(a))


def test_rmsnorm_matches_library():
    x = RNG.standard_normal(300)
    g = RNG.standard_normal(300).astype(np.float32)
    ref = F.rms_norm(torch.from_numpy(x), (300,), torch.from_numpy(g).double(), eps=1e-5).numpy()
    np.testing.assert_allclose(rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-14)


def test_rmsnorm_closed_form():
    # constant vector c with unit gains -> c / sqrt(c^2 + eps) everywhere
    x = np.full(64, 3.0)
    out = rmsnorm(x, np.ones(64), 1e-5)
    np.testing.assert_allclose(out, 3.0 / np.sqrt(9.0 + 1e-5), rtol=1e-14)
    # eps matters: a zero vector stays zero, no NaN
    assert np.all(rmsnorm(np.zeros(8), np.ones(8), 1e-5) == 0.0)


def test_rope_is_complex_rotation():
    # rotate-half pairing (i, i+hd/2): z_i = a_i + i b_i is multiplied by exp(i p theta_i)
    hd, heads, pos, base = 64, 3, 37, 10000.0
    v = RNG.standard_normal(heads * hd)
    out = rope(v, heads, hd, pos, base).reshape(heads, hd)
    vin = v.reshape(heads, hd)
    z = vin[:, :hd // 2] + 1j * vin[:, hd // 2:]
    theta = base ** (-2.0 * np.arange(hd // 2) / hd)
    zr = z * np.exp(1j * pos * theta)[None, :]
    np.testing.assert_allclose(out[:, :hd // 2], zr.real, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out[:, hd // 2:], zr.imag, rtol=1e-12, atol=1e-13)


def test_rope_identity_norm_and_relative_position():
    hd, base = 128, 500000.0
    q = RNG.standard_normal(hd)
    k = RNG.standard_normal(hd)
    np.testing.assert_array_equal(rope(q, 1, hd, 0, base), q)            # p = 0: identity
    np.testing.assert_allclose(np.linalg.norm(rope(q, 1, hd, 911, base)), np.linalg.norm(q), rtol=1e-12)
    # the score depends only on the distance between the two positions
    a = rope(q, 1, hd, 50, base) @ rope(k, 1, hd, 20, base)
    b = rope(q, 1, hd, 1030, base) @ rope(k, 1, hd, 1000, base)
    np.testing.assert_allclose(a, b, rtol=1e-9)


@pytest.mark.parametrize("nq,nkv,hd,T", [(4, 2, 64, 23), (8, 8, 32, 5), (32, 8, 128, 70), (4, 2, 64, 1)])
def test_attention_matches_library(nq, nkv, hd, T):
    q = RNG.standard_normal(nq * hd)
    K = RNG.standard_normal((T, nkv * hd)).astype(np.float32)
    V = RNG.standard_normal((T, nkv * hd)).astype(np.float32)
    o = attention(q, K, V, nq, nkv, hd).reshape(nq, hd)
    tq = torch.from_numpy(q).reshape(1, nq, 1, hd)
    tk = torch.from_numpy(K).double().reshape(T, nkv, hd).permute(1, 0, 2)[None]
    tv = torch.from_numpy(V).double().reshape(T, nkv, hd).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, enable_gqa=True)[0, :, 0].numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    nq, nkv, hd, T = 4, 2, 16, 9
    q = RNG.standard_normal(nq * hd)
    V = RNG.standard_normal((T, nkv * hd)).astype(np.float32)
    # all keys equal -> uniform weights -> output is the mean of V per kv head
    K = np.tile(RNG.standard_normal((1, nkv * hd)).astype(np.float32), (T, 1))
    o = attention(q, K, V, nq, nkv, hd).reshape(nq, hd)
    mean = V.astype(np.float64).mean(axis=0).reshape(nkv, hd)
    for i in range(nq):
        np.testing.assert_allclose(o[i], mean[i // 2], rtol=1e-12, atol=1e-14)
    # one position: output is that value row, whatever q is
    o1 = attention(q, K[:1], V[:1], nq, nkv, hd).reshape(nq, hd)
    for i in range(nq):
        np.testing.assert_allclose(o1[i], V[0].reshape(nkv, hd)[i // 2], rtol=1e-14)
    # huge scores do not overflow (max is subtracted)
    big = attention(q * 1e4, RNG.standard_normal((T, nkv * hd)).astype(np.float32), V, nq, nkv, hd)
    assert np.all(np.isfinite(big))


def test_swiglu_matches_library():
    g = RNG.standard_normal(1000) * 4
    u = RNG.standard_normal(1000)
    out = np.empty(1000)
    ro.lib().orc_swiglu(_p(g), _p(u), 1000, _p(out))
    ref = (F.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-15)


def test_cosine_closed_forms():
    h = RNG.standard_normal(256)
    g = RNG.standard_normal(256)
    assert cosine(h, h) == pytest.approx(1.0, abs=1e-15)
    assert cosine(h, -h) == pytest.approx(-1.0, abs=1e-15)
    e0, e1 = np.eye(256)[0], np.eye(256)[1]
    assert cosine(e0, e1) == 0.0
    assert cosine(e0 + e1, e0) == pytest.approx(1 / np.sqrt(2), rel=1e-14)
    assert cosine(3.5 * h, 0.01 * g) == pytest.approx(cosine(h, g), rel=1e-12)   # scale invariance
    assert cosine(h, g) == pytest.approx(cosine(g, h), rel=1e-15)                # symmetry
    assert cosine(np.zeros(256), h) == 0.0 and cosine(h, np.zeros(256)) == 0.0   # zero-norm rule
    ref = F.cosine_similarity(torch.from_numpy(h)[None], torch.from_numpy(g)[None]).item()
    assert cosine(h, g) == pytest.approx(ref, rel=1e-12)
    for _ in range(200):                                                         # Cauchy-Schwarz
        a = RNG.standard_normal(8) * 10 ** RNG.uniform(-3, 3)
        assert -1.0 <= cosine(a, a * (1 + 1e-16)) <= 1.0


def test_bf16_rounding_matches_library():
    x = np.concatenate([RNG.standard_normal(5000) * 10 ** RNG.uniform(-6, 6, 5000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38]]).astype(np.float32)
    ours = np.array([ro.lib().orc_f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    np.testing.assert_array_equal(ours, ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert ro.lib().orc_f32_to_bf16(1.00390625) == 0x3F80
    assert ro.lib().orc_f32_to_bf16(1.01171875) == 0x3F82


def test_f16_rounding_bit_exact_with_torch():
    """The oracle's fp32 -> IEEE half rounding (the FP16 KV cache) against torch's conversion:
    random values over the whole range, ties, subnormals, the overflow boundary, signs."""
    import ctypes
    L = ro.lib()
    rng = np.random.default_rng(3)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 70000.0, -65520.0, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0000001, 2.0 ** -14, 2.0 ** -14 * 0.9999, 6.1e-5, 5.96e-8, 3e-8, 1e-10,
            1.00048828125, 1.00146484375, 2049.0, 2051.0, 0.333333, 1e-3, 1023.5, 1024.5]
    vals += list(rng.standard_normal(4000).astype(np.float32) * np.float32(0.7))
    vals += list((rng.standard_normal(2000) * 10.0 ** rng.uniform(-9, 5, 2000)).astype(np.float32))
    # exact ties: halfway between two neighbouring halves
    h = rng.integers(0x0001, 0x7bff, 2000).astype(np.uint16)
    lo = torch.from_numpy(h.view(np.int16)).view(torch.float16).to(torch.float32)
    hi = torch.from_numpy((h + 1).astype(np.uint16).view(np.int16)).view(torch.float16).to(torch.float32)
    vals += list(((lo + hi) / 2).numpy())
    v = np.array(vals, dtype=np.float32)
    v = np.concatenate([v, -v])
    want = torch.from_numpy(v).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.orc_f32_to_f16(ctypes.c_float(float(x))) for x in v], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)
    back = np.array([L.orc_f16_to_f32(int(x)) for x in want[:5000]], dtype=np.float32)
    ref = torch.from_numpy(want[:5000].view(np.int16)).view(torch.float16).to(torch.float32).numpy()
    np.testing.assert_array_equal(back, ref)
