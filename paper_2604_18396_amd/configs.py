"""Model / workload shapes for the early-exit decode path.

Only shapes and knobs live here: no arithmetic of the method.  The five
workloads are the ones the benchmark definition names (tiny fp32, 1B-shape
bf16, 8B-shape bf16 short context, 8B long context, 8B ragged batch 16).

Notation follows the paper (method section, "Inference with Seamless Exit"):
L blocks numbered 1..L, h(0) is the embedding, the exit position e of a token
is the number of backbone blocks it executed, L_s is the entry layer of the
Exit River (smallest allowed exit position), tau the threshold of Eq. 1.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

DTYPE_F32 = 0
DTYPE_BF16 = 1
KV_SAME = 0
KV_F16 = 1


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float
    dtype: int            # DTYPE_F32: fp32 weights + cache; DTYPE_BF16: bf16 weights + cache
    max_seq: int
    min_exit_layer: int   # L_s
    tau: float
    river_group: int = 64
    kv_dtype: int = 0     # KV-cache storage: 0 = the weight dtype, 1 = fp16 (bf16 models only)

    @property
    def params_per_block(self) -> int:
        d, f = self.d_model, self.d_ffn
        q = self.n_q_heads * self.head_dim
        kv = self.n_kv_heads * self.head_dim
        return d * q + 2 * d * kv + q * d + 3 * d * f

    def with_(self, **kw) -> "ModelConfig":
        return replace(self, **kw)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    prompt_len: int
    decode_steps: int
    batch: int
    exit_mode: str        # "threshold" (Eq. 1) or "forced" (seeded schedule)
    seed_weights: int
    seed_prompt: int
    seed_exits: int


TINY = ModelConfig("tiny-fp32", 4, 256, 4, 2, 64, 688, 512, 10000.0, 1e-5,
                   DTYPE_F32, 64, 2, 0.9)
LLAMA_1B = ModelConfig("llama-1b-shape", 16, 2048, 32, 8, 64, 8192, 32000, 10000.0, 1e-5,
                       DTYPE_BF16, 512, 4, 2.0)
LLAMA_8B = ModelConfig("llama-8b-shape", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, 1e-5,
                       DTYPE_BF16, 1024, 8, 2.0)

C1 = Workload("C1-tiny-fp32", TINY, 16, 32, 1, "threshold", 1001, 2001, 0)
C2 = Workload("C2-1b-bf16", LLAMA_1B, 256, 256, 1, "forced", 1002, 2002, 3002)
C3 = Workload("C3-8b-bf16-ctx512", LLAMA_8B, 512, 512, 1, "forced", 1003, 2003, 3003)
C4 = Workload("C4-8b-bf16-ctx4096", LLAMA_8B.with_(max_seq=5120), 4096, 1024, 1, "forced",
              1003, 2004, 3004)
C5 = Workload("C5-8b-bf16-batch16", LLAMA_8B.with_(max_seq=1280), 1024, 256, 16, "forced",
              1003, 2005, 3005)

WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5)}

# order of the seven quantised matrices of a block, used by every interface
MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def matrix_shape(cfg: ModelConfig, name: str) -> tuple[int, int]:
    """[out, in] shape (nn.Linear orientation, row-major) of one block matrix."""
    q = cfg.n_q_heads * cfg.head_dim
    kv = cfg.n_kv_heads * cfg.head_dim
    return {
        "wq": (q, cfg.d_model), "wk": (kv, cfg.d_model), "wv": (kv, cfg.d_model),
        "wo": (cfg.d_model, q), "w_gate": (cfg.d_ffn, cfg.d_model),
        "w_up": (cfg.d_ffn, cfg.d_model), "w_down": (cfg.d_model, cfg.d_ffn),
    }[name]
