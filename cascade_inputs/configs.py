"""The five workload configurations (shapes only; no arithmetic)."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class LayerConfig:
    name: str
    dtype: str          # "f32" or "bf16" (bf16 storage, fp32 accumulation)
    d_model: int        # D
    n_heads: int        # H
    n_kv_heads: int     # H_KV
    head_dim: int       # d
    d_ff: int           # f
    norm: str           # "layernorm" | "rmsnorm"
    act: str            # "gelu" | "gelu_tanh" | "swiglu"
    rope: bool
    rope_theta: float
    bias: bool          # linear biases and norm bias present
    eps: float
    batch: int          # B
    seq_len: int        # N
    n_shards: int       # beta (R = S sharding: alpha = beta)
    assignment: str     # "perm" | "contiguous" | "roundrobin"
    sigma: float        # std of weight entries
    index: int          # position in the benchmark's config list
    norm_placement: str = "pre"   # "pre": x + f(norm(x)) blocks; "post": norm(x + f(x)) blocks (BERT-shaped)

    @property
    def scale(self) -> float:
        return self.head_dim ** -0.5

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


CONFIGS = {
    "C1": LayerConfig("C1-tiny-f32", "f32", 64, 4, 4, 16, 256, "layernorm", "gelu", False, 0.0, True,
                      1e-5, 1, 128, 4, "perm", 0.02, 0),
    "C2": LayerConfig("C2-gpt2-small-bf16", "bf16", 768, 12, 12, 64, 3072, "layernorm", "gelu", False, 0.0,
                      True, 1e-5, 4, 1024, 8, "contiguous", 0.02, 1),
    "C3": LayerConfig("C3-llama3-8b-bf16", "bf16", 4096, 32, 8, 128, 14336, "rmsnorm", "swiglu", True,
                      500000.0, False, 1e-5, 1, 2048, 16, "perm", 0.02, 2),
    "C4": LayerConfig("C4-llama3-8b-long-bf16", "bf16", 4096, 32, 8, 128, 14336, "rmsnorm", "swiglu", True,
                      500000.0, False, 1e-5, 1, 8192, 64, "roundrobin", 0.02, 3),
    "C5": LayerConfig("C5-llama3-70b-bf16", "bf16", 8192, 64, 8, 128, 28672, "rmsnorm", "swiglu", True,
                      500000.0, False, 1e-5, 1, 4096, 32, "perm", 0.015, 4),
}


def get_config(key: str) -> LayerConfig:
    return CONFIGS[key]
