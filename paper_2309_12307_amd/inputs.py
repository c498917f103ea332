"""Seeded synthetic inputs for S2-Attn, shared by the tests, the bench and the
oracle-side checks.  Holds no attention arithmetic: only random draws, the
benchmark shape table and host-side bf16 rounding of the drawn values.

The configurations stand in for post-RoPE Llama2 activations (the paper's
fine-tuning data and weights are not available): iid N(0,1) values, drawn with
numpy.random.default_rng(1000 + c) for configuration c in the order q, k, v, dO.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class S2Config:
    name: str
    index: int
    dtype: str      # "f32" or "bf16"
    B: int
    N: int
    H: int
    Hkv: int
    D: int
    G: int

    @property
    def shift(self) -> int:
        return self.G // 2

    @property
    def seed(self) -> int:
        return 1000 + self.index


CONFIGS = {
    "C1": S2Config("C1", 1, "f32", 1, 256, 4, 4, 64, 64),
    "C2": S2Config("C2", 2, "bf16", 1, 8192, 32, 32, 128, 2048),
    "C3": S2Config("C3", 3, "bf16", 1, 32768, 32, 32, 128, 8192),
    "C4": S2Config("C4", 4, "bf16", 1, 32768, 64, 8, 128, 8192),
    "C5": S2Config("C5", 5, "bf16", 1, 102400, 32, 32, 128, 25600),
}


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def draw(shape_q, shape_kv, seed: int):
    """q, k, v, dO as float32 standard normals, in that draw order."""
    rng = np.random.default_rng(seed)
    q = rng.standard_normal(shape_q, dtype=np.float32)
    k = rng.standard_normal(shape_kv, dtype=np.float32)
    v = rng.standard_normal(shape_kv, dtype=np.float32)
    do = rng.standard_normal(shape_q, dtype=np.float32)
    return q, k, v, do


def make_inputs(B, N, H, Hkv, D, seed, dtype="f32"):
    """Returns dict with float32 arrays q, k, v, do.  For dtype "bf16" the values
    are already rounded to bf16 (so both the GPU, via `*_bits`, and the oracle,
    via the float32 up-casts, see identical numbers)."""
    q, k, v, do = draw((B, N, H, D), (B, N, Hkv, D), seed)
    out = {}
    if dtype == "bf16":
        for name, x in (("q", q), ("k", k), ("v", v), ("do", do)):
            bits = round_to_bf16_bits(x)
            out[name + "_bits"] = bits
            out[name] = bf16_bits_to_f32(bits)
    elif dtype == "f32":
        out.update(q=q, k=k, v=v, do=do)
    else:
        raise ValueError(dtype)
    return out


def make_config_inputs(cfg: S2Config):
    return make_inputs(cfg.B, cfg.N, cfg.H, cfg.Hkv, cfg.D, cfg.seed, cfg.dtype)
