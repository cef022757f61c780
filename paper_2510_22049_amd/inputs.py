"""Seeded synthetic inputs for the five workload configurations.

This module only draws random numbers, rounds them to a storage dtype and lays
out the jagged batch.  It holds none of the method's arithmetic, so both the CPU
oracle's tests and the HIP path's tests may use it without sharing any code of
the computation itself.

The shapes follow the workloads the paper talks about (Sec. 5.1, Table 1:
industrial histories with mean 7k / max 16k items; the abstract and Sec. 1:
"10k to 100k" and lifelong histories of up to a million items; Sec. 5.2.2 and
App. D: 64-128 seeds or "a few hundred", d in 32..256, 4 heads).  None of the
paper's datasets is reproduced: only lengths and tensor shapes are borrowed.

Every tensor gets its own counter-based stream keyed by (config, tensor name,
user index), so a single user of a large configuration can be regenerated alone.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field

import numpy as np

SEED = 0


@dataclass(frozen=True)
class Config:
    """One workload configuration (shapes only; no arithmetic)."""

    index: int
    name: str
    B: int            # users
    d: int            # model width
    H: int            # heads
    S: int            # virtual queries / summary tokens
    dtype: str        # "f32" or "bf16"
    C: int = 0        # candidates per user (0 = stage 1 only)
    layers: int = 1   # stacked summarization layers
    d_ff: int = 0     # inner width of the gated block between layers
    length_rule: str = "fixed"
    length_args: tuple = field(default_factory=tuple)


CONFIGS = {
    1: Config(1, "tiny", B=1, d=64, H=1, S=16, dtype="f32", C=32,
              length_rule="fixed", length_args=(1024,)),
    2: Config(2, "jagged", B=64, d=128, H=4, S=256, dtype="bf16",
              length_rule="lognormal", length_args=(8000.0, 1.0, 1000, 100000)),
    3: Config(3, "lifelong", B=8, d=128, H=4, S=256, dtype="bf16",
              length_rule="fixed", length_args=(1_000_000,)),
    4: Config(4, "serving", B=1024, d=128, H=4, S=256, dtype="bf16", C=512,
              length_rule="none"),
    5: Config(5, "end_to_end", B=256, d=256, H=8, S=512, dtype="bf16", C=256,
              layers=2, d_ff=512, length_rule="uniform",
              length_args=(10000, 100000)),
}


def stream(config: int, tensor: str, user: int = 0) -> np.random.Generator:
    """Independent generator for (config, tensor, user); seed 0 everywhere."""
    key = zlib.crc32(tensor.encode("ascii"))
    ss = np.random.SeedSequence([SEED, int(config), key, int(user)])
    return np.random.Generator(np.random.Philox(ss))


def lengths(cfg: Config, B: int | None = None) -> np.ndarray:
    """History length of each user, int64[B]."""
    B = cfg.B if B is None else B
    g = stream(cfg.index, "lengths")
    if cfg.length_rule == "fixed":
        return np.full(B, cfg.length_args[0], dtype=np.int64)
    if cfg.length_rule == "lognormal":
        median, sigma, lo, hi = cfg.length_args
        raw = np.exp(g.normal(np.log(median), sigma, size=B))
        return np.clip(np.rint(raw), lo, hi).astype(np.int64)
    if cfg.length_rule == "uniform":
        lo, hi = cfg.length_args
        return g.integers(lo, hi + 1, size=B, dtype=np.int64)
    raise ValueError(f"config {cfg.index} has no history")


def offsets_from_lengths(lens) -> np.ndarray:
    """Exclusive prefix sum: int64[B+1], offsets[0] = 0, offsets[B] = N."""
    lens = np.asarray(lens, dtype=np.int64)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    return off


# ---------------------------------------------------------------- dtypes

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round values to the storage dtype and return them widened to fp32."""
    if dtype == "bf16":
        return from_bf16_bits(to_bf16_bits(x))
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def normal(g: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    """N(0, std^2) draws rounded to the storage dtype (returned as fp32)."""
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return round_to(x, dtype)


# ---------------------------------------------------------------- tensors

def history_user(cfg: Config, user: int, length: int) -> np.ndarray:
    """Item embeddings of one user, [length, d], ~N(0,1), storage-rounded."""
    return normal(stream(cfg.index, "history", user), (int(length), cfg.d), 1.0, cfg.dtype)


def history(cfg: Config, lens) -> np.ndarray:
    """Packed jagged history [N, d]; rows of user b are offsets[b]..offsets[b+1]-1."""
    off = offsets_from_lengths(lens)
    out = np.empty((int(off[-1]), cfg.d), dtype=np.float32)
    for b, L in enumerate(lens):
        out[off[b]:off[b + 1]] = history_user(cfg, b, int(L))
    return out


def virtual_queries(cfg: Config) -> np.ndarray:
    """Learned seeds shared by all users, [S, d], ~N(0,1)."""
    return normal(stream(cfg.index, "virtual_queries"), (cfg.S, cfg.d), 1.0, cfg.dtype)


def projection(cfg: Config, name: str, layer: int = 0) -> np.ndarray:
    """W_k or W_v of a layer, [d, d] (input rows, output columns), ~N(0, 1/d)."""
    g = stream(cfg.index, f"{name}{layer}")
    return normal(g, (cfg.d, cfg.d), cfg.d ** -0.5, cfg.dtype)


def ffn_weights(cfg: Config, layer: int = 0):
    """W_g, W_u [d, d_ff] and W_o [d_ff, d] of the gated block, ~N(0, 1/fan_in)."""
    d, f = cfg.d, cfg.d_ff
    wg = normal(stream(cfg.index, f"W_g{layer}"), (d, f), d ** -0.5, cfg.dtype)
    wu = normal(stream(cfg.index, f"W_u{layer}"), (d, f), d ** -0.5, cfg.dtype)
    wo = normal(stream(cfg.index, f"W_o{layer}"), (f, d), f ** -0.5, cfg.dtype)
    return wg, wu, wo


def candidates_user(cfg: Config, user: int, C: int | None = None) -> np.ndarray:
    """Candidate item embeddings of one user, [C, d], ~N(0,1)."""
    C = cfg.C if C is None else C
    return normal(stream(cfg.index, "candidates", user), (C, cfg.d), 1.0, cfg.dtype)


def summaries_user(cfg: Config, user: int) -> np.ndarray:
    """Stand-in cached summary tokens of one user, [S, d], ~N(0,1) (serving config)."""
    return normal(stream(cfg.index, "summaries", user), (cfg.S, cfg.d), 1.0, cfg.dtype)
