"""Thin ctypes binding of libriver.so (include/river.h).

Argument marshalling only: every step of the decode path runs in the library's HIP
kernels.  torch is used for device memory and the stream.  If the library has not
been built, loading raises: there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from . import build as _build
from .configs import MATRICES, ModelConfig

RIVER_OK, RIVER_EINVAL, RIVER_ENOSPC, RIVER_ESTATE, RIVER_EHIP = 0, -1, -2, -3, -4
EXEC_KERNELS, EXEC_PERSISTENT = 0, 1
DBG_HIDDEN, DBG_LOGITS, DBG_KCACHE, DBG_VCACHE, DBG_TRACE, DBG_BATCH_HIDDEN, DBG_BATCH_LOGITS = 0, 1, 2, 3, 4, 5, 6
EXIT_PER_SEQUENCE, EXIT_BATCH_MIN = 0, 1

EXPORTS = ("river_quantize_w4", "river_workspace_bytes", "river_create", "river_create_static", "river_prefill",
           "river_decode_step", "river_decode_batch", "river_read_batch_records", "river_read_records",
           "river_rewind", "river_position", "river_seq_position",
           "river_get_debug", "river_fill_cache", "river_last_error", "river_destroy")


class RiverError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"river error {code}: {msg}")
        self.code = code


class river_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("min_exit_layer", C.c_int32),
                ("tau", C.c_float), ("river_bits", C.c_int32), ("river_group", C.c_int32),
                ("exec_mode", C.c_int32), ("spin_limit", C.c_int32), ("prefill_gemm_min_tokens", C.c_int32),
                ("batch_exit_rule", C.c_int32), ("kv_dtype", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class river_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, _PP) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up",
                                   "w_down")]


class river_qweights(C.Structure):
    _fields_ = [("codes", _PP * 7), ("scale", _PP * 7), ("zero", _PP * 7)]


_lib = None


def load():
    """Load libriver.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("RIVER_LIB_PATH", _build.LIB)      # e.g. the diagnostics build
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first "
                          "(python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(path)
    L.river_quantize_w4.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.river_workspace_bytes.argtypes = [C.POINTER(river_config)]
    L.river_workspace_bytes.restype = C.c_size_t
    L.river_create.argtypes = [C.POINTER(river_config), C.POINTER(river_weights),
                               C.POINTER(river_qweights), C.c_void_p, C.c_size_t, C.c_void_p,
                               C.POINTER(C.c_void_p)]
    L.river_create_static.argtypes = L.river_create.argtypes
    L.river_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                C.POINTER(C.c_int32), C.c_void_p]
    L.river_decode_step.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
    L.river_decode_batch.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p]
    L.river_read_batch_records.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.river_seq_position.argtypes = [C.c_void_p, C.c_int32]
    L.river_read_records.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.river_rewind.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.river_position.argtypes = [C.c_void_p]
    L.river_get_debug.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t]
    L.river_fill_cache.argtypes = [C.c_void_p, C.c_int32]
    L.river_last_error.argtypes = [C.c_void_p]
    L.river_last_error.restype = C.c_char_p
    L.river_destroy.argtypes = [C.c_void_p]
    _lib = L
    return L


def default_exec_mode(cfg: ModelConfig) -> int:
    """One launch per token where the library offers it (bf16), else one launch per phase."""
    return EXEC_PERSISTENT if cfg.dtype == 1 else EXEC_KERNELS


def make_config(cfg: ModelConfig, exec_mode: int | None = None, spin_limit: int = 0,
                prefill_gemm_min_tokens: int = 0, max_batch: int = 1, batch_exit_rule: int = 0) -> river_config:
    if exec_mode is None:
        exec_mode = default_exec_mode(cfg)
    return river_config(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        cfg.d_ffn, cfg.vocab, cfg.rope_base, cfg.rms_eps, cfg.dtype, max_batch, cfg.max_seq,
                        cfg.min_exit_layer, cfg.tau, 4, cfg.river_group, exec_mode, spin_limit,
                        prefill_gemm_min_tokens, batch_exit_rule, cfg.kv_dtype)


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def river_quantize_w4(w: torch.Tensor, group: int):
    """Device tensor [rows, cols] (fp32 / bf16) -> (codes u8 [rows, cols/2], scale, zero)."""
    assert w.is_cuda and w.is_contiguous() and w.dim() == 2
    rows, cols = w.shape
    gpr = -(-cols // group)
    codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=w.device)
    scale = torch.empty((rows, gpr), dtype=w.dtype, device=w.device)
    zero = torch.empty((rows, gpr), dtype=w.dtype, device=w.device)
    dt = 1 if w.dtype == torch.bfloat16 else 0
    rc = load().river_quantize_w4(w.data_ptr(), rows, cols, group, dt, codes.data_ptr(),
                                  scale.data_ptr(), zero.data_ptr(), _stream_ptr())
    if rc:
        raise RiverError(rc, "river_quantize_w4")
    return codes, scale, zero


def upload_weights(weights: dict, device="cuda:0") -> dict:
    """CPU weight dict (inputs.make_weights) -> same structure on the device."""
    out = {k: weights[k].to(device) for k in ("tok_emb", "final_norm", "lm_head")}
    out["layers"] = [{k: v.to(device) for k, v in blk.items()} for blk in weights["layers"]]
    return out


def offload_backbone(dev_weights: dict, from_block: int) -> dict:
    """Backbone Offloading: the seven matrices of backbone blocks from_block+1..L (1-based: the
    blocks a token only reaches when its exit position exceeds from_block) are moved out of
    HBM into pinned host memory, which the GPU reads in place over the host link when a token
    does reach them; norm gains, embedding, head and the whole river stay in HBM.  Build the
    river first (quantize_river reads the matrices on the device).  Returns a new weight dict."""
    out = {k: dev_weights[k] for k in ("tok_emb", "final_norm", "lm_head")}
    out["layers"] = []
    for l, blk in enumerate(dev_weights["layers"]):
        if l < from_block:
            out["layers"].append(blk)
            continue
        nb = {}
        for k, v in blk.items():
            if k in MATRICES:
                host = torch.empty(v.shape, dtype=v.dtype, pin_memory=True)
                host.copy_(v)
                nb[k] = host
            else:
                nb[k] = v
        out["layers"].append(nb)
    torch.cuda.synchronize()
    return out


def quantize_river(cfg: ModelConfig, dev_weights: dict) -> list:
    """River construction on the device for every block (list of {name: (codes, scale, zero)})."""
    return [{m: river_quantize_w4(blk[m], cfg.river_group) for m in MATRICES}
            for blk in dev_weights["layers"]]


class River:
    """One decode context (river_create .. river_destroy)."""

    def __init__(self, cfg: ModelConfig, dev_weights: dict, dev_river: list | None,
                 exec_mode: int | None = None, spin_limit: int = 0, static_scratch: bool = False,
                 prefill_gemm_min_tokens: int = 0, max_batch: int = 1, batch_exit_rule: int = 0):
        """static_scratch=True goes through river_create_static (no device allocation inside
        the library: activations and barrier counters in the library's static device array)."""
        L = load()
        self.cfg = cfg
        self._c = make_config(cfg, exec_mode, spin_limit, prefill_gemm_min_tokens, max_batch, batch_exit_rule)
        self.max_batch = max_batch
        self._keep = [dev_weights, dev_river]
        n = cfg.n_layers
        w = river_weights()
        w.tok_emb = dev_weights["tok_emb"].data_ptr()
        w.final_norm = dev_weights["final_norm"].data_ptr()
        w.lm_head = dev_weights["lm_head"].data_ptr()
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            arr = (C.c_void_p * n)(*[blk[name].data_ptr() for blk in dev_weights["layers"]])
            self._keep.append(arr)
            setattr(w, name, C.cast(arr, _PP))
        q = None
        if dev_river is not None:
            q = river_qweights()
            for j, m in enumerate(MATRICES):
                for k, field in enumerate(("codes", "scale", "zero")):
                    arr = (C.c_void_p * n)(*[(r[m][k].data_ptr() if r is not None else None)
                                             for r in dev_river])
                    self._keep.append(arr)
                    getattr(q, field)[j] = C.cast(arr, _PP)
        nbytes = L.river_workspace_bytes(C.byref(self._c))
        if nbytes == 0:
            raise RiverError(RIVER_EINVAL, "invalid configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev_weights["tok_emb"].device)
        self.workspace_bytes = nbytes
        h = C.c_void_p()
        create = L.river_create_static if static_scratch else L.river_create
        rc = create(C.byref(self._c), C.byref(w), C.byref(q) if q is not None else None,
                    self.workspace.data_ptr(), nbytes, _stream_ptr(), C.byref(h))
        if rc:
            raise RiverError(rc, L.river_last_error(None).decode())
        self._h = h

    def _check(self, rc: int):
        if rc:
            raise RiverError(rc, load().river_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None):
            load().river_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens, exit_layer: int | None = None, out_logits: torch.Tensor | None = None,
                seq: int = 0) -> int:
        """Prefill phase at the unified depth exit_layer (None: the full depth L).
        out_logits: optional device fp32 [vocab] tensor that receives the last position's logits.
        seq: the sequence of a batched context."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        out = C.c_int32()
        if out_logits is not None:
            assert out_logits.is_cuda and out_logits.dtype == torch.float32 and out_logits.is_contiguous()
            assert out_logits.numel() == self.cfg.vocab
        self._check(load().river_prefill(self._h, seq, t.ctypes.data, len(t),
                                         -1 if exit_layer is None else int(exit_layer), C.byref(out),
                                         out_logits.data_ptr() if out_logits is not None else None))
        return out.value

    def decode_step(self, token: int | None = None, forced_exit: int | None = None, sync: bool = True):
        """sync=True -> (next_token, exit_position, sims[L]); sync=False queues the step only."""
        tin = C.byref(C.c_int32(int(token))) if token is not None else None
        fe = C.byref(C.c_int32(int(forced_exit))) if forced_exit is not None else None
        if not sync:
            self._check(load().river_decode_step(self._h, tin, fe, None, None, None))
            return None
        tok, e = C.c_int32(), C.c_int32()
        sims = np.empty(self.cfg.n_layers, dtype=np.float32)
        self._check(load().river_decode_step(self._h, tin, fe, C.byref(tok), C.byref(e),
                                             sims.ctypes.data))
        return tok.value, e.value, sims

    def decode_batch(self, n_seq: int, tokens=None, forced_exits=None, sync: bool = True):
        """One step of a batched context.  sync=True -> (tokens[n], exit_positions[n], sims[n, L])."""
        tin = np.ascontiguousarray(tokens, dtype=np.int32) if tokens is not None else None
        fe = (np.ascontiguousarray([-1 if f is None else int(f) for f in forced_exits], dtype=np.int32)
              if forced_exits is not None else None)
        a = tin.ctypes.data if tin is not None else None
        b = fe.ctypes.data if fe is not None else None
        if not sync:
            self._check(load().river_decode_batch(self._h, n_seq, a, b, None, None, None))
            return None
        toks = np.empty(n_seq, dtype=np.int32)
        es = np.empty(n_seq, dtype=np.int32)
        sims = np.empty((n_seq, self.cfg.n_layers), dtype=np.float32)
        self._check(load().river_decode_batch(self._h, n_seq, a, b, toks.ctypes.data, es.ctypes.data,
                                              sims.ctypes.data))
        return toks, es, sims

    def read_batch_records(self, n_steps: int, n_seq: int):
        toks = np.empty((n_steps, n_seq), dtype=np.int32)
        es = np.empty((n_steps, n_seq), dtype=np.int32)
        self._check(load().river_read_batch_records(self._h, n_steps, n_seq, toks.ctypes.data, es.ctypes.data))
        return toks, es

    def seq_pos(self, seq: int) -> int:
        return load().river_seq_position(self._h, seq)

    def batch_hidden(self) -> np.ndarray:
        """[L+1, max_batch, d] hidden states of the last batched step."""
        out = np.empty((self.cfg.n_layers + 1, self.max_batch, self.cfg.d_model), dtype=np.float32)
        self._check(load().river_get_debug(self._h, DBG_BATCH_HIDDEN, out.ctypes.data, out.nbytes))
        return out

    def batch_logits(self) -> np.ndarray:
        out = np.empty((self.max_batch, self.cfg.vocab), dtype=np.float32)
        self._check(load().river_get_debug(self._h, DBG_BATCH_LOGITS, out.ctypes.data, out.nbytes))
        return out

    def read_records(self, n: int):
        toks = np.empty(n, dtype=np.int32)
        es = np.empty(n, dtype=np.int32)
        sims = np.empty((n, self.cfg.n_layers), dtype=np.float32)
        self._check(load().river_read_records(self._h, n, toks.ctypes.data, es.ctypes.data,
                                              sims.ctypes.data))
        return toks, es, sims

    def rewind(self, new_len: int, seq: int = 0):
        self._check(load().river_rewind(self._h, seq, new_len))

    @property
    def pos(self) -> int:
        return load().river_position(self._h)

    def hidden(self) -> np.ndarray:
        out = np.empty((self.cfg.n_layers + 1, self.cfg.d_model), dtype=np.float32)
        self._check(load().river_get_debug(self._h, DBG_HIDDEN, out.ctypes.data, out.nbytes))
        return out

    def logits(self) -> np.ndarray:
        out = np.empty(self.cfg.vocab, dtype=np.float32)
        self._check(load().river_get_debug(self._h, DBG_LOGITS, out.ctypes.data, out.nbytes))
        return out

    def _cache(self, what) -> np.ndarray:
        c = self.cfg
        kvd = c.n_kv_heads * c.head_dim
        shape = (c.n_layers, c.max_seq, kvd) if self.max_batch == 1 else (self.max_batch, c.n_layers, c.max_seq, kvd)
        if c.dtype == 1:
            raw = np.empty(shape, dtype=np.uint16)
            self._check(load().river_get_debug(self._h, what, raw.ctypes.data, raw.nbytes))
            if c.kv_dtype == 1:
                return raw.view(np.float16).astype(np.float32)         # IEEE half words -> fp32 values
            return (raw.astype(np.uint32) << 16).view(np.float32)      # bf16 words -> fp32 values
        raw = np.empty(shape, dtype=np.float32)
        self._check(load().river_get_debug(self._h, what, raw.ctypes.data, raw.nbytes))
        return raw

    def kcache(self) -> np.ndarray:
        return self._cache(DBG_KCACHE)

    def vcache(self) -> np.ndarray:
        return self._cache(DBG_VCACHE)

    def trace(self, workgroups: int) -> np.ndarray:
        """[5L, 2, workgroups] barrier arrive/release device times (diagnostics build only)."""
        n = 5 * self.cfg.n_layers * 2 * workgroups
        out = np.empty(n + 64, dtype=np.uint64)
        self._check(load().river_get_debug(self._h, DBG_TRACE, out.ctypes.data, out.nbytes))
        self.marks = out[n:].astype(np.int64)
        return out[:n].reshape(5 * self.cfg.n_layers, 2, workgroups)

    def fill_cache(self, byte: int):
        self._check(load().river_fill_cache(self._h, byte))


# The C entry points under their own names (the class above is the same calls with
# the context kept in an object).
def river_create(cfg, dev_weights, dev_river, exec_mode=None, spin_limit=0) -> River:
    return River(cfg, dev_weights, dev_river, exec_mode, spin_limit)


def river_create_static(cfg, dev_weights, dev_river, exec_mode=None, spin_limit=0) -> River:
    return River(cfg, dev_weights, dev_river, exec_mode, spin_limit, static_scratch=True)


def river_prefill(ctx: River, tokens, exit_layer=None, out_logits=None) -> int:
    return ctx.prefill(tokens, exit_layer, out_logits)


def river_decode_step(ctx: River, token=None, forced_exit=None, sync=True):
    return ctx.decode_step(token, forced_exit, sync)


def river_decode_batch(ctx: River, n_seq: int, tokens=None, forced_exits=None, sync=True):
    return ctx.decode_batch(n_seq, tokens, forced_exits, sync)


def river_read_batch_records(ctx: River, n_steps: int, n_seq: int):
    return ctx.read_batch_records(n_steps, n_seq)


def river_read_records(ctx: River, n: int):
    return ctx.read_records(n)


def river_rewind(ctx: River, new_len: int):
    ctx.rewind(new_len)


def river_destroy(ctx: River):
    ctx.close()
