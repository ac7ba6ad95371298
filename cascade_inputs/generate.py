"""Seeded tensor and assignment generators.  Plain draws and bf16 rounding only."""
import numpy as np

from .configs import LayerConfig

BASE_SEED = 0xC45CADE


def config_seed(cfg: LayerConfig) -> int:
    return BASE_SEED + cfg.index


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    return bf16_bits_to_f32(bf16_bits(x))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_assignment(kind: str, seq_len: int, n_shards: int, seed: int) -> np.ndarray:
    """token_to_shard[N] (int32) for one of the assignment patterns of the workloads.

    "perm": a seeded random permutation cut into n_shards equal consecutive chunks;
    "contiguous": blocks of N/n_shards neighbouring tokens;
    "roundrobin": token t goes to shard t mod n_shards;
    "ragged": seeded uniformly random shard per token (unequal, possibly empty shards).
    """
    t = np.arange(seq_len)
    if kind == "contiguous":
        size = -(-seq_len // n_shards)
        a = t // size
    elif kind == "roundrobin":
        a = t % n_shards
    elif kind == "perm":
        rng = np.random.Generator(np.random.PCG64(seed ^ 0x5A4D))
        p = rng.permutation(seq_len)
        size = -(-seq_len // n_shards)
        a = np.empty(seq_len, dtype=np.int64)
        a[p] = t // size
    elif kind == "ragged":
        rng = np.random.Generator(np.random.PCG64(seed ^ 0x7A66))
        a = rng.integers(0, n_shards, size=seq_len)
    else:
        raise ValueError(kind)
    return a.astype(np.int32)


def _normal(rng, shape, std, as_bf16):
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return round_to_bf16(x) if as_bf16 else x


def make_hidden(cfg: LayerConfig, seed: int = None) -> np.ndarray:
    """Hidden states h[B, N, D] ~ N(0, 1), float32 (on the bf16 grid for bf16 configs)."""
    seed = config_seed(cfg) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x1111))
    return _normal(rng, (cfg.batch, cfg.seq_len, cfg.d_model), 1.0, cfg.dtype == "bf16")


def make_layer_weights(cfg: LayerConfig, seed: int = None) -> dict:
    """Layer parameters as float32 arrays, [out_features, in_features] for matrices.

    Matrices ~ N(0, sigma); biases ~ N(0, sigma) when cfg.bias; norm gains 1 + N(0, sigma);
    norm biases ~ N(0, sigma) for LayerNorm.  bf16 configs are rounded onto the bf16 grid.
    """
    seed = config_seed(cfg) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x2222))
    bf = cfg.dtype == "bf16"
    D, H, Hkv, d, f, s = cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ff, cfg.sigma
    w = {}
    w["wq"] = _normal(rng, (H * d, D), s, bf)
    w["wk"] = _normal(rng, (Hkv * d, D), s, bf)
    w["wv"] = _normal(rng, (Hkv * d, D), s, bf)
    w["wo"] = _normal(rng, (D, H * d), s, bf)
    if cfg.act == "swiglu":
        w["w_gate"] = _normal(rng, (f, D), s, bf)
    w["w_up"] = _normal(rng, (f, D), s, bf)
    w["w_down"] = _normal(rng, (D, f), s, bf)
    w["norm1_g"] = (1.0 + _normal(rng, (D,), s, False)).astype(np.float32)
    w["norm2_g"] = (1.0 + _normal(rng, (D,), s, False)).astype(np.float32)
    if bf:
        w["norm1_g"] = round_to_bf16(w["norm1_g"])
        w["norm2_g"] = round_to_bf16(w["norm2_g"])
    if cfg.norm == "layernorm":
        w["norm1_b"] = _normal(rng, (D,), s, bf)
        w["norm2_b"] = _normal(rng, (D,), s, bf)
    if cfg.bias:
        w["bq"] = _normal(rng, (H * d,), s, bf)
        w["bk"] = _normal(rng, (Hkv * d,), s, bf)
        w["bv"] = _normal(rng, (Hkv * d,), s, bf)
        w["bo"] = _normal(rng, (D,), s, bf)
        w["b_up"] = _normal(rng, (f,), s, bf)
        w["b_down"] = _normal(rng, (D,), s, bf)
    return w


def make_head_weights(cfg: LayerConfig, vocab: int, seed: int = None) -> dict:
    """Closing norm and vocabulary projection [vocab, d_model], drawn like the layer parameters."""
    seed = config_seed(cfg) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x4444))
    bf = cfg.dtype == "bf16"
    head = {"w_vocab": _normal(rng, (vocab, cfg.d_model), cfg.sigma, bf),
            "norm_g": (1.0 + _normal(rng, (cfg.d_model,), cfg.sigma, False)).astype(np.float32)}
    if bf:
        head["norm_g"] = round_to_bf16(head["norm_g"])
    if cfg.norm == "layernorm":
        head["norm_b"] = _normal(rng, (cfg.d_model,), cfg.sigma, bf)
    return head
