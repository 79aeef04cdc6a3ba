"""The plain definition of what early-exit decode with a KV-Shared Exit River computes.

TEST INFRASTRUCTURE ONLY.  numpy, fp64, no KV cache, for tiny shapes.

Definition (River-LLM method section: shared KV addressing of the exit layers,
serial river after the exit, Eq. 1): given tokens x_0..x_t and exit positions
e_0..e_t, position j uses the backbone matrices W_l in blocks l <= e_j and the
river twins W^_l in blocks l > e_j.  The whole causal transformer is run over
positions 0..t from scratch; position j attends to the keys/values of positions
0..j of the same block, whichever matrices produced them.  The output of step t
is argmax(W_head . RMSNorm(h_t^(L))).  In threshold mode e_j is the smallest l
in [L_s, L-1] whose similarity cos(h_j^(l-1), h_j^(l)) exceeds tau, else L,
found on this same run.

This is the object the incremental, cached algorithm in river_oracle.c must
reproduce; it also carries an independent numpy statement of the 4-bit format.
"""
from __future__ import annotations

import numpy as np
import torch

MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def to_f64(t) -> np.ndarray:
    if isinstance(t, torch.Tensor):
        return t.to(torch.float64).numpy()
    return np.asarray(t, dtype=np.float64)


def round_to(v: np.ndarray, dtype: int, kv_dtype: int = 0) -> np.ndarray:
    """fp64 values -> values of the cache's storage type (kv_dtype 1: IEEE half; else the
    weight dtype: 0 fp32, 1 bf16), round-to-nearest-even."""
    t = torch.from_numpy(np.ascontiguousarray(v)).to(torch.float32)
    if kv_dtype == 1:
        t = t.to(torch.float16)
    elif dtype == 1:
        t = t.to(torch.bfloat16)
    return t.to(torch.float64).numpy()


def quantize_w4(w: torch.Tensor, group: int):
    """4-bit asymmetric round-to-nearest, groups of `group` consecutive input elements per
    output row (a shorter last group when group does not divide cols); fp32 arithmetic;
    scale and zero stored in w's dtype; two codes per byte, even index in the low nibble."""
    rows, cols = w.shape
    st = w.dtype
    w32 = w.to(torch.float32)
    scales, zeros, qs = [], [], []
    for c0 in range(0, cols, group):
        g = w32[:, c0:c0 + group]
        mn = g.amin(dim=1, keepdim=True)
        mx = g.amax(dim=1, keepdim=True)
        scale = torch.where(mx > mn, (mx - mn) / 15.0, torch.ones_like(mx)).to(st)
        s32 = scale.to(torch.float32)
        zero = (-mn / s32).to(st)
        z32 = zero.to(torch.float32)
        qs.append(torch.clamp(torch.round(g / s32 + z32), 0, 15).to(torch.uint8))
        scales.append(scale)
        zeros.append(zero)
    q = torch.cat(qs, dim=1)
    codes = (q[:, 0::2] | (q[:, 1::2] << 4)).contiguous()
    return codes, torch.cat(scales, dim=1).contiguous(), torch.cat(zeros, dim=1).contiguous()


def dequantize_w4(codes: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor, group: int) -> np.ndarray:
    """w^ = (q - zero) * scale evaluated in fp32, returned as fp64."""
    rows, cols = codes.shape[0], codes.shape[1] * 2
    q = torch.stack([codes & 15, codes >> 4], dim=2).reshape(rows, cols).to(torch.float32)
    s = scale.to(torch.float32).repeat_interleave(group, dim=1)[:, :cols]
    z = zero.to(torch.float32).repeat_interleave(group, dim=1)[:, :cols]
    return ((q - z) * s).to(torch.float64).numpy()


def _rmsnorm(x, g, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def _rope(v, positions, hd, base):
    """v: [T, heads, hd]; rotate-half pairing (i, i+hd/2), angle p * base^(-2i/hd)."""
    half = hd // 2
    inv = base ** (-2.0 * np.arange(half) / hd)
    ang = positions[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def run(cfg, weights: dict, river: list | None, tokens, exits=None):
    """Full no-cache run over all positions.

    exits: None -> every position decides by Eq. 1 (cfg.tau, cfg.min_exit_layer);
    otherwise one entry per token: an exit position to force (L = full depth, as
    used for prompt positions) or None to let Eq. 1 decide for that token.
    Returns dict(hidden [T, L+1, d], logits [T, V], tokens [T], exits [T], sims [T, L]).
    """
    L, d, nq, nkv, hd = cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    # eps, tau and the RoPE base are single-precision configuration fields: use those values
    eps, tau = float(np.float32(cfg.rms_eps)), float(np.float32(cfg.tau))
    base = float(np.float32(cfg.rope_base))
    T = len(tokens)
    pos = np.arange(T, dtype=np.float64)
    emb = to_f64(weights["tok_emb"])
    h = emb[np.asarray(tokens)]                       # [T, d]
    hidden = np.zeros((T, L + 1, d))
    hidden[:, 0] = h
    sims = np.full((T, L), np.nan)
    e = np.full(T, L, dtype=np.int64)
    exited = np.zeros(T, dtype=bool)
    forced = [None] * T if exits is None else list(exits)
    for j in range(T):
        if forced[j] == 0:
            exited[j], e[j] = True, 0
    causal = np.tril(np.ones((T, T), dtype=bool))
    for l in range(1, L + 1):
        blk = weights["layers"][l - 1]
        Wb = {m: to_f64(blk[m]) for m in MATRICES}
        Wr = None
        if exited.any():
            q = river[l - 1]
            Wr = {m: dequantize_w4(*q[m], cfg.river_group) for m in MATRICES}

        def mm(name, x):                              # per-position choice of matrices
            y = x @ Wb[name].T
            if Wr is not None:
                y[exited] = x[exited] @ Wr[name].T
            return y

        x = _rmsnorm(h, to_f64(blk["attn_norm"]), eps)
        qv = _rope(mm("wq", x).reshape(T, nq, hd), pos, hd, base)
        kv = _rope(mm("wk", x).reshape(T, nkv, hd), pos, hd, base)
        vv = mm("wv", x).reshape(T, nkv, hd)
        kv = round_to(kv, cfg.dtype, getattr(cfg, "kv_dtype", 0))   # what the cache stores
        vv = round_to(vv, cfg.dtype, getattr(cfg, "kv_dtype", 0))
        rep = nq // nkv
        o = np.zeros((T, nq, hd))
        for i in range(nq):
            sc = qv[:, i] @ kv[:, i // rep].T / np.sqrt(hd)
            sc = np.where(causal, sc, -np.inf)
            sc = np.exp(sc - sc.max(axis=1, keepdims=True))
            a = sc / sc.sum(axis=1, keepdims=True)
            o[:, i] = a @ vv[:, i // rep]
        h1 = h + mm("wo", o.reshape(T, nq * hd))
        y = _rmsnorm(h1, to_f64(blk["ffn_norm"]), eps)
        g = mm("w_gate", y)
        u = mm("w_up", y)
        h2 = h1 + mm("w_down", g / (1.0 + np.exp(-g)) * u)
        for j in range(T):
            if exited[j]:
                continue
            na, nb = np.linalg.norm(h[j]), np.linalg.norm(h2[j])
            s = 0.0 if na == 0 or nb == 0 else float(np.clip(h[j] @ h2[j] / (na * nb), -1, 1))
            sims[j, l - 1] = s
            if cfg.min_exit_layer <= l < L:
                if (forced[j] is None and s > tau) or forced[j] == l:
                    exited[j], e[j] = True, l
        h = h2
        hidden[:, l] = h
    xn = _rmsnorm(h, to_f64(weights["final_norm"]), eps)
    logits = xn @ to_f64(weights["lm_head"]).T
    return {"hidden": hidden, "logits": logits, "tokens": logits.argmax(axis=1),
            "exits": e, "sims": sims}
