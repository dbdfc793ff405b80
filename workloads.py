"""Seeded synthetic inputs and the five benchmark shapes.

Shared by the tests, the smoke check and the benchmark so that the HIP path and the
fp64 oracle see the same bits.  Holds NO arithmetic of the method: only shapes, a
seeded normal generator, and rounding of the generated values to the storage type.

The shapes stand in for the long-sequence LLaMA2-7B activations of the paper's
evaluation (Sec. "Experiment Setup": D=4096, H=32, H_kv=8, head_dim 128, sequences of
128K..1M tokens): values are N(0,1)*0.5 rounded once to bf16; the kernel's cost does
not depend on the values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class RingConfig:
    name: str
    cp: int            # context-parallel degree being simulated
    w: int             # inner ring size (w == cp or 1: plain ring)
    rank: int          # simulated device
    hq: int            # local q heads
    hkv: int           # local kv heads
    d: int             # head dim
    c: int             # half-chunk length; local tokens L = 2c, total S = 2*cp*c
    dtype: str         # "bf16" | "fp16" | "fp32"
    sigma: float       # values ~ N(0,1) * sigma
    seed: int

    @property
    def L(self) -> int:
        return 2 * self.c

    @property
    def S(self) -> int:
        return 2 * self.cp * self.c

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    def shrunk(self, c: int) -> "RingConfig":
        """Same grid, heads and head_dim with a shorter chunk (full-tensor parity)."""
        return replace(self, c=c, name=f"{self.name}@c{c}")

    def on_rank(self, rank: int) -> "RingConfig":
        return replace(self, rank=rank, name=f"{self.name}@r{rank}")


CONFIGS = [
    RingConfig("tiny_fp32", cp=4, w=4, rank=0, hq=2, hkv=2, d=64, c=128, dtype="fp32", sigma=1.0, seed=1000),
    RingConfig("mha7b_32k", cp=8, w=8, rank=0, hq=8, hkv=8, d=128, c=2048, dtype="bf16", sigma=0.5, seed=1001),
    RingConfig("gqa7b_128k", cp=8, w=8, rank=0, hq=4, hkv=1, d=128, c=8192, dtype="bf16", sigma=0.5, seed=1002),
    RingConfig("dring_256k", cp=16, w=4, rank=0, hq=8, hkv=8, d=128, c=8192, dtype="bf16", sigma=0.5, seed=1003),
    RingConfig("long_1m", cp=32, w=32, rank=0, hq=4, hkv=1, d=128, c=16384, dtype="bf16", sigma=0.5, seed=1004),
]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are exactly representable in bf16
    (round to nearest, ties to even on the upper 16 bits)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) >> 16).astype(np.uint32) << 16
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-exact fp32 values, as uint16 (raw storage for the device)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-exact"
    return (u >> 16).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _normal(rng, shape, sigma, dtype):
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float32)   # round to nearest even
    return round_to_bf16(x) if dtype == "bf16" else x


def make_inputs(cfg: RingConfig) -> dict:
    """q, d_out: the simulated device's rows [hq, L, d]; k_all, v_all: every key of
    the sequence in natural order [hkv, S, d].  fp32 arrays (bf16- or fp16-exact for the 16-bit types)."""
    rng = np.random.Generator(np.random.Philox(cfg.seed))
    return {
        "q": _normal(rng, (cfg.hq, cfg.L, cfg.d), cfg.sigma, cfg.dtype),
        "d_out": _normal(rng, (cfg.hq, cfg.L, cfg.d), cfg.sigma, cfg.dtype),
        "k_all": _normal(rng, (cfg.hkv, cfg.S, cfg.d), cfg.sigma, cfg.dtype),
        "v_all": _normal(rng, (cfg.hkv, cfg.S, cfg.d), cfg.sigma, cfg.dtype),
    }


def gather_chunks(x_all: np.ndarray, chunk_ids, c: int) -> np.ndarray:
    """Rows of the listed global chunks of x_all [h, S, d], concatenated: [h, len*c, d]."""
    return np.concatenate([x_all[:, i * c:(i + 1) * c] for i in chunk_ids], axis=1)
