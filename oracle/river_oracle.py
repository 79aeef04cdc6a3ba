"""ctypes front end of the C oracle (oracle/river_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, never by the product package.  Argument
marshalling only; every number comes out of the C file.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("max_seq", C.c_int32), ("min_exit_layer", C.c_int32), ("tau", C.c_float),
                ("river_group", C.c_int32), ("kv_dtype", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class _QMat(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scale", C.c_void_p), ("zero", C.c_void_p)]


class _QLayer(C.Structure):
    _fields_ = [("m", _QMat * 7)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        L = _lib
        L.orc_quantize_w4.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_dequantize_w4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                        C.c_int, C.c_int, C.c_void_p]
        L.orc_create.argtypes = [C.POINTER(_Cfg), C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.POINTER(_Layer), C.POINTER(_QLayer), C.POINTER(C.c_void_p)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_destroy.restype = None
        L.orc_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32)]
        L.orc_decode_step.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                      C.POINTER(C.c_int32), C.c_void_p]
        L.orc_rewind.argtypes = [C.c_void_p, C.c_int]
        L.orc_pos.argtypes = [C.c_void_p]
        L.orc_block.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_embed.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.orc_head.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        L.orc_advance.argtypes = [C.c_void_p]
        for name, rt in (("orc_hidden", C.c_double), ("orc_logits", C.c_double),
                         ("orc_kcache", C.c_float), ("orc_vcache", C.c_float),
                         ("orc_written", C.c_uint8)):
            f = getattr(L, name)
            f.argtypes = [C.c_void_p]
            f.restype = C.POINTER(rt)
        L.orc_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_void_p]
        L.orc_rmsnorm.restype = None
        L.orc_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_double]
        L.orc_rope.restype = None
        L.orc_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                    C.c_int, C.c_void_p]
        L.orc_attention.restype = None
        L.orc_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.orc_swiglu.restype = None
        L.orc_cosine.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.orc_cosine.restype = C.c_double
        L.orc_f32_to_bf16.argtypes = [C.c_float]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        L.orc_f16_to_f32.restype = C.c_float
    return _lib


def _ptr(t) -> int:
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous() and t.device.type == "cpu"
        return t.data_ptr()
    assert t.flags["C_CONTIGUOUS"]
    return t.ctypes.data


def quantize_w4(w: torch.Tensor, group: int):
    """Oracle river quantiser.  w: CPU tensor [rows, cols] fp32 or bf16.
    Returns (codes uint8 [rows, cols/2], scale [rows, cols/group], zero [...]) in w's dtype."""
    rows, cols = w.shape
    dt = 1 if w.dtype == torch.bfloat16 else 0
    codes = torch.empty((rows, cols // 2), dtype=torch.uint8)
    gpr = (cols + group - 1) // group
    scale = torch.empty((rows, gpr), dtype=w.dtype)
    zero = torch.empty((rows, gpr), dtype=w.dtype)
    rc = lib().orc_quantize_w4(_ptr(w), rows, cols, group, dt, _ptr(codes), _ptr(scale), _ptr(zero))
    if rc:
        raise ValueError(f"orc_quantize_w4 failed: {rc}")
    return codes, scale, zero


def dequantize_w4(codes, scale, zero, group: int) -> np.ndarray:
    rows, cols = codes.shape[0], codes.shape[1] * 2
    dt = 1 if scale.dtype == torch.bfloat16 else 0
    out = np.empty((rows, cols), dtype=np.float64)
    lib().orc_dequantize_w4(_ptr(codes), _ptr(scale), _ptr(zero), rows, cols, group, dt, _ptr(out))
    return out


def quantize_river(cfg, weights: dict) -> list:
    """Quantise the seven matrices of every block l > L_s... (all blocks here: a twin for every
    block costs nothing in the oracle and lets tests force any depth).  Returns a list of
    {name: (codes, scale, zero)} per layer (None where the backbone layer is None)."""
    out = []
    for blk in weights["layers"]:
        out.append(None if blk is None else
                   {m: quantize_w4(blk[m], cfg.river_group) for m in MATRICES})
    return out


class Oracle:
    """Incremental (cached) early-exit decode, as the paper's method section defines it."""

    def __init__(self, cfg, weights: dict, river: list | None):
        L = lib()
        self.cfg = cfg
        self._keep = (weights, river)
        c = _Cfg(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                 cfg.vocab, cfg.rope_base, cfg.rms_eps, cfg.dtype, cfg.max_seq, cfg.min_exit_layer,
                 cfg.tau, cfg.river_group, getattr(cfg, "kv_dtype", 0))
        layers = (_Layer * cfg.n_layers)()
        for i, blk in enumerate(weights["layers"]):
            for n, _ in _Layer._fields_:
                setattr(layers[i], n, _ptr(blk[n]))
        qlayers = (_QLayer * cfg.n_layers)()
        if river is not None:
            for i, q in enumerate(river):
                if q is None:
                    continue
                for j, m in enumerate(MATRICES):
                    qlayers[i].m[j].codes = _ptr(q[m][0])
                    qlayers[i].m[j].scale = _ptr(q[m][1])
                    qlayers[i].m[j].zero = _ptr(q[m][2])
        h = C.c_void_p()
        rc = L.orc_create(C.byref(c), _ptr(weights["tok_emb"]), _ptr(weights["final_norm"]),
                          _ptr(weights["lm_head"]), layers, qlayers, C.byref(h))
        if rc:
            raise ValueError(f"orc_create failed: {rc}")
        self._h = h

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens, exit_layer: int | None = None) -> int:
        """Prefill phase at the unified depth exit_layer (None: the full depth L)."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        out = C.c_int32()
        rc = lib().orc_prefill(self._h, _ptr(t), len(t), -1 if exit_layer is None else int(exit_layer),
                               C.byref(out))
        if rc:
            raise ValueError(f"orc_prefill failed: {rc}")
        return out.value

    def decode_step(self, token: int, forced_exit: int | None = None):
        """Returns (next_token, exit_position, sims[L] with NaN for river blocks)."""
        tok, e = C.c_int32(), C.c_int32()
        sims = np.empty(self.cfg.n_layers, dtype=np.float64)
        rc = lib().orc_decode_step(self._h, int(token), -1 if forced_exit is None else int(forced_exit),
                                   C.byref(tok), C.byref(e), _ptr(sims))
        if rc:
            raise ValueError(f"orc_decode_step failed: {rc}")
        return tok.value, e.value, sims

    def rewind(self, new_len: int):
        rc = lib().orc_rewind(self._h, new_len)
        if rc:
            raise ValueError(f"orc_rewind failed: {rc}")

    @property
    def pos(self) -> int:
        return lib().orc_pos(self._h)

    def hidden(self) -> np.ndarray:
        """[L+1, d] hidden states h(0..L) of the last token processed."""
        n = (self.cfg.n_layers + 1) * self.cfg.d_model
        return np.ctypeslib.as_array(lib().orc_hidden(self._h), (n,)).reshape(
            self.cfg.n_layers + 1, self.cfg.d_model).copy()

    def logits(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().orc_logits(self._h), (self.cfg.vocab,)).copy()

    def _cache(self, fn) -> np.ndarray:
        c = self.cfg
        kvd = c.n_kv_heads * c.head_dim
        return np.ctypeslib.as_array(fn(self._h), (c.n_layers * c.max_seq * kvd,)).reshape(
            c.n_layers, c.max_seq, kvd)

    def kcache(self) -> np.ndarray:
        return self._cache(lib().orc_kcache)

    def vcache(self) -> np.ndarray:
        return self._cache(lib().orc_vcache)

    def written(self) -> np.ndarray:
        c = self.cfg
        return np.ctypeslib.as_array(lib().orc_written(self._h), (c.n_layers * c.max_seq,)).reshape(
            c.n_layers, c.max_seq)

    def embed(self, token: int) -> np.ndarray:
        h = np.empty(self.cfg.d_model, dtype=np.float64)
        if lib().orc_embed(self._h, int(token), _ptr(h)):
            raise ValueError("orc_embed failed")
        return h

    def head(self, h: np.ndarray) -> int:
        """Final norm + LM head on h (logits() afterwards); returns the greedy token."""
        h = np.ascontiguousarray(h, dtype=np.float64)
        tok = C.c_int32()
        if lib().orc_head(self._h, _ptr(h), C.byref(tok)):
            raise ValueError("orc_head failed")
        return tok.value

    def advance(self):
        if lib().orc_advance(self._h):
            raise ValueError("orc_advance failed")

    def block(self, layer1: int, pos: int, river: bool, h: np.ndarray) -> np.ndarray:
        h = np.ascontiguousarray(h, dtype=np.float64)
        out = np.empty_like(h)
        rc = lib().orc_block(self._h, layer1, pos, int(river), _ptr(h), _ptr(out))
        if rc:
            raise ValueError(f"orc_block failed: {rc}")
        return out
