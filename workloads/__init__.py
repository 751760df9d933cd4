"""Seeded synthetic inputs shared by the oracle-side and the HIP-side callers.

This module holds no arithmetic of the method: it only draws random tensors,
rounds them to the storage type the kernels read, and names the benchmark
configurations.  Both the tests and the benchmark hand the *same* arrays to
the CPU oracle and to the HIP library.

The paper's workload is LLaMA3-8B attention on 16K-token book text (Sec. 6.1);
neither the weights nor the corpus are available, so the inputs are synthetic
tensors of that model's attention shape (32 query heads, 8 KV heads,
head_dim 128).

Every (tensor, batch, head) slice has its own generator stream, so one
(batch, KV-head) slice of a large configuration can be produced without
materialising the rest.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_TENSOR_ID = {"q": 0, "k": 1, "v": 2, "do": 3, "mu_q": 4, "mu_k": 5}


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "f32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    chunk_len: int
    seed: int
    rope_like: bool = False
    spaco_t: int = 0    # number of selected chunks (0: SeCO only)

    @property
    def n_chunks(self):
        return -(-self.seq_len // self.chunk_len)

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.head_dim))


CONFIGS = {
    "cfg1": Config("cfg1", "f32", 1, 4, 4, 64, 1024, 256, seed=0),
    "cfg2": Config("cfg2", "bf16", 1, 32, 8, 128, 16384, 1024, seed=1),
    "cfg3": Config("cfg3", "bf16", 1, 32, 8, 128, 32768, 2048, seed=2, spaco_t=4),
    "cfg4": Config("cfg4", "bf16", 1, 32, 8, 128, 65536, 2048, seed=3, spaco_t=8),
    "cfg5_c512": Config("cfg5_c512", "bf16", 2, 32, 8, 128, 32768, 512, seed=4, rope_like=True, spaco_t=16),
    "cfg5_c1024": Config("cfg5_c1024", "bf16", 2, 32, 8, 128, 32768, 1024, seed=4, rope_like=True, spaco_t=8),
    "cfg5_c2048": Config("cfg5_c2048", "bf16", 2, 32, 8, 128, 32768, 2048, seed=4, rope_like=True, spaco_t=4),
    "cfg5_c4096": Config("cfg5_c4096", "bf16", 2, 32, 8, 128, 32768, 4096, seed=4, rope_like=True, spaco_t=2),
    # the paper's own chunk-size sweep (Sec. 6.3: 16K tokens, chunks of 32 .. 512, SpaCO with t = 8)
    "small_c32": Config("small_c32", "bf16", 1, 32, 8, 128, 16384, 32, seed=5, spaco_t=8),
    "small_c64": Config("small_c64", "bf16", 1, 32, 8, 128, 16384, 64, seed=5, spaco_t=8),
    "small_c128": Config("small_c128", "bf16", 1, 32, 8, 128, 16384, 128, seed=5, spaco_t=8),
    "small_c256": Config("small_c256", "bf16", 1, 32, 8, 128, 16384, 256, seed=5, spaco_t=8),
    "small_c512": Config("small_c512", "bf16", 1, 32, 8, 128, 16384, 512, seed=5, spaco_t=8),
    # longer contexts than the paper trains on (its limit is 16K tokens on 24 GB), chunks sized for this GPU
    "cfg2_b2": Config("cfg2_b2", "bf16", 2, 32, 8, 128, 16384, 1024, seed=1),   # cfg2 with two sequences per call
    "long_128k": Config("long_128k", "bf16", 1, 32, 8, 128, 131072, 4096, seed=6, spaco_t=8),
    "long_256k": Config("long_256k", "bf16", 1, 32, 8, 128, 262144, 8192, seed=6, spaco_t=8),
}


# ---- storage rounding ------------------------------------------------------

def f32_to_bf16_bits(x):
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(x, dtype):
    """fp32 array whose values are exactly representable in `dtype`."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    if dtype == "f32":
        return x
    raise ValueError(f"unknown dtype {dtype!r}")


# ---- generators ------------------------------------------------------------

def _normal(seed, tensor, b, h, shape):
    rng = np.random.default_rng([int(seed), _TENSOR_ID[tensor], int(b), int(h)])
    return rng.standard_normal(shape, dtype=np.float32)


def _rotate(x, positions, base=500000.0):
    """Rotary rotation of consecutive dimension pairs (2i, 2i+1) by angle pos * base^(-2i/D)."""
    n, d = x.shape
    inv = base ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    ang = positions[:, None].astype(np.float64) * inv[None, :]
    c, s = np.cos(ang), np.sin(ang)
    x = x.astype(np.float64)
    out = np.empty_like(x)
    out[:, 0::2] = x[:, 0::2] * c - x[:, 1::2] * s
    out[:, 1::2] = x[:, 0::2] * s + x[:, 1::2] * c
    return out.astype(np.float32)


def head_slice(cfg: Config, tensor: str, b: int, h: int):
    """[N, D] fp32 slice of tensor `tensor` in {"q","k","v","do"} for batch b, head h.

    Plain configs: i.i.d. N(0,1).  RoPE-like configs: Q and K are
    rotate(pos) applied to (mu_head + g), g ~ N(0,1), mu_head a fixed vector of
    norm 2 per head; V and dO stay N(0,1).
    Values are rounded to the configuration's storage type.
    """
    n, d = cfg.seq_len, cfg.head_dim
    x = _normal(cfg.seed, tensor, b, h, (n, d))
    if cfg.rope_like and tensor in ("q", "k"):
        mu = _normal(cfg.seed, "mu_" + tensor, 0, h, (d,))
        mu *= np.float32(2.0) / np.linalg.norm(mu).astype(np.float32)
        x = _rotate(x + mu[None, :], np.arange(n))
    return round_to(x, cfg.dtype)


def kv_group(cfg: Config, b: int, kv_head: int):
    """All inputs of one independent (batch, KV-head) unit.

    returns dict with q, do [G, N, D] and k, v [N, D] (fp32, storage-rounded).
    """
    g = cfg.n_q_heads // cfg.n_kv_heads
    heads = range(kv_head * g, (kv_head + 1) * g)
    return {
        "q": np.stack([head_slice(cfg, "q", b, h) for h in heads]),
        "do": np.stack([head_slice(cfg, "do", b, h) for h in heads]),
        "k": head_slice(cfg, "k", b, kv_head),
        "v": head_slice(cfg, "v", b, kv_head),
    }


def full_layer(cfg: Config):
    """Whole-layer tensors: q, do [B,Hq,N,D]; k, v [B,Hkv,N,D] (fp32, storage-rounded)."""
    def build(tensor, nh):
        return np.stack([np.stack([head_slice(cfg, tensor, b, h) for h in range(nh)])
                         for b in range(cfg.batch)])
    return {
        "q": build("q", cfg.n_q_heads),
        "k": build("k", cfg.n_kv_heads),
        "v": build("v", cfg.n_kv_heads),
        "do": build("do", cfg.n_q_heads),
    }


def small_layer(seed, B, Hq, Hkv, N, D, dtype="f32"):
    """Small ad-hoc layer for unit tests: dict q, k, v, do (fp32, storage-rounded)."""
    cfg = Config("adhoc", dtype, B, Hq, Hkv, D, N, N, seed=seed)
    return full_layer(cfg)
