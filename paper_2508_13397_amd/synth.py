"""Seeded synthetic rank buffers, shaped like the paper's workloads (large gradient-style
all-reduce buffers of 32-bit floats; Results section: 2^27 .. 2^29 floats per GPU).

This module only draws random numbers.  It holds none of the all-reduce arithmetic, so both
the GPU path and the CPU oracle can be fed from it.  Rank r draws from its own counter-based
Philox stream keyed by BASE_SEED + r, so any rank's buffer can be regenerated alone.

Distributions:
  "int_pm1000"   int32, uniform integers in [-1000, 1000]
  "uniform_pm1"  float32, uniform in [-1, 1)
  "normal"       float32, N(0, 1)
  "normal_bf16"  N(0, sigma^2 = 1e-2) drawn in float32, narrowed to bf16 by torch's CPU
                 conversion (a library routine, independent of the code under test);
                 returned as uint16 bit patterns
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 250813397

DISTS = ("int_pm1000", "uniform_pm1", "normal", "normal_bf16")


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16) through torch's CPU conversion."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def rank_buffer(rank: int, n: int, dist: str, seed: int = BASE_SEED) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=seed + rank))
    if dist == "int_pm1000":
        return rng.integers(-1000, 1001, size=n, dtype=np.int32)
    if dist == "uniform_pm1":
        x = rng.random(n, dtype=np.float32)
        x *= np.float32(2.0)
        x -= np.float32(1.0)
        return x
    if dist == "normal":
        return rng.standard_normal(n, dtype=np.float32)
    if dist == "normal_bf16":
        x = rng.standard_normal(n, dtype=np.float32)
        x *= np.float32(0.1)
        return to_bf16_bits(x)
    raise ValueError(f"unknown distribution {dist!r}; expected one of {DISTS}")


def make_inputs(P: int, n: int, dist: str, seed: int = BASE_SEED, workers: int = 8) -> np.ndarray:
    """[P, n] array, row r = rank r's buffer."""
    first = rank_buffer(0, n, dist, seed)
    out = np.empty((P, n), dtype=first.dtype)
    out[0] = first

    def fill(r):
        out[r] = rank_buffer(r, n, dist, seed)

    if P > 1:
        if workers > 1 and n * P >= (1 << 22):
            with ThreadPoolExecutor(max_workers=workers) as ex:
                list(ex.map(fill, range(1, P)))
        else:
            for r in range(1, P):
                fill(r)
    return out


def order_sensitive_f32(P: int, n: int) -> np.ndarray:
    """float32 buffers for which the order of a left-to-right sum shows in the result: large
    values of both signs next to small ones, different per rank and element (deterministic,
    no random draws)."""
    r = np.arange(P, dtype=np.uint64)[:, None]
    i = np.arange(n, dtype=np.uint64)[None, :]
    h = (r * np.uint64(2654435761) + i * np.uint64(40503) + np.uint64(12345)) % np.uint64(1 << 32)
    h = (h ^ (h >> np.uint64(13))) * np.uint64(1274126177) % np.uint64(1 << 32)
    expo = np.array([0.0, 9.0, 17.0, 26.0])[((h >> np.uint64(7)) % np.uint64(4)).astype(np.int64)]
    sign = np.where((h >> np.uint64(3)) % np.uint64(2) == 0, 1.0, -1.0)
    frac = 1.0 + ((h >> np.uint64(11)) % np.uint64(1 << 20)).astype(np.float64) / float(1 << 20)
    return (sign * frac * np.exp2(expo)).astype(np.float32)
