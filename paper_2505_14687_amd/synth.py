"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This module holds no attention or grouping arithmetic: it only names the benchmark
workloads (token grid, group shape, heads, head_dim, dtype) and draws Q, K, V ~ N(0,1)
from counter-free numpy generators, one independent stream per (tensor, head), so that a
single head of a large workload can be regenerated without producing the rest.

bf16 tensors are handed out as uint16 bit patterns (float32 rounded to nearest-even and
truncated to its upper 16 bits); every consumer decodes them with its own code.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    grid: Tuple[int, ...]          # token grid, row-major, last dim fastest
    group: Tuple[int, ...]         # tokens per group along each grid dim
    batch: int
    heads: int
    head_dim: int
    dtype: str                     # "bf16" or "f32"
    seed: int
    patterns: Dict[str, Tuple[str, Tuple[int, ...]]] = field(default_factory=dict)

    @property
    def n_tokens(self) -> int:
        return int(np.prod(self.grid))

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


# pattern label -> (pattern name, per-axis radius; ignored by the cross patterns)
WORKLOADS: Dict[str, Workload] = {
    "tiny2d": Workload("tiny2d", (32, 32), (8, 8), 1, 2, 64, "f32", 1001,
                       {"B3": ("block", (1, 1)), "X": ("cross", (0, 0))}),
    "img1024": Workload("img1024", (64, 64), (16, 16), 1, 24, 128, "bf16", 1002,
                        {"B3": ("block", (1, 1)), "X": ("cross", (0, 0))}),
    "img2048": Workload("img2048", (128, 128), (16, 16), 1, 24, 128, "bf16", 1003,
                        {"B3": ("block", (1, 1)), "B5": ("block", (2, 2)),
                         "X": ("cross", (0, 0)), "dense": ("dense", (0, 0))}),
    "img8192": Workload("img8192", (512, 512), (16, 16), 1, 24, 128, "bf16", 1004,
                        {"B3": ("block", (1, 1)), "X": ("cross", (0, 0))}),
    "video": Workload("video", (30, 48, 80), (2, 8, 8), 1, 24, 128, "bf16", 1005,
                      {"B3": ("block", (1, 1, 1)), "X": ("cross", (0, 0, 0)),
                       "Xplanes": ("cross_planes", (0, 0, 0))}),
    # --- beyond the five benchmark configs: the paper's own video shape (Sec. 4.2: 32x48x80 latent
    # tokens, groups 4x8x8) and the group-size / radius ablation of its appendix at 512x512 tokens
    "video_paper": Workload("video_paper", (32, 48, 80), (4, 8, 8), 1, 24, 128, "bf16", 1006,
                            {"B3": ("block", (1, 1, 1)), "X": ("cross", (0, 0, 0)),
                             "Xplanes": ("cross_planes", (0, 0, 0))}),
    "img8192_g8": Workload("img8192_g8", (512, 512), (8, 8), 1, 24, 128, "bf16", 1007,
                           {"B3": ("block", (1, 1)), "B5": ("block", (2, 2)), "B7": ("block", (3, 3)),
                            "X": ("cross", (0, 0))}),
    "img8192_g32": Workload("img8192_g32", (512, 512), (32, 32), 1, 24, 128, "bf16", 1008,
                            {"B3": ("block", (1, 1)), "X": ("cross", (0, 0))}),
    "img8192_b2": Workload("img8192_b2", (512, 512), (16, 16), 1, 24, 128, "bf16", 1004,
                           {"B5": ("block", (2, 2))}),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def _head_stream(seed: int, tensor: int, b: int, h: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, tensor, b, h]))


def head_normal(seed: int, tensor: int, b: int, h: int, n: int, d: int,
                gain: float = 1.0) -> np.ndarray:
    """float32 [n, d] ~ N(0, gain^2) for one (tensor, batch, head); tensor 0/1/2 = Q/K/V."""
    x = _head_stream(seed, tensor, b, h).standard_normal((n, d), dtype=np.float32)
    if gain != 1.0:
        x *= np.float32(gain)
    return x


def make_qkv(batch: int, heads: int, n: int, d: int, dtype: str, seed: int,
             q_gain: float = 1.0, threads: int = 8):
    """Q, K, V of shape [batch, heads, n, d].

    dtype "f32": float32 arrays.  dtype "bf16": uint16 arrays of bf16 bit patterns.  dtype "f16":
    float16 arrays (float32 rounded to nearest-even).
    q_gain scales Q before rounding (a gain of 4 makes the softmax peaked).
    """
    out_dt = {"f32": np.float32, "bf16": np.uint16, "f16": np.float16}[dtype]
    out = [np.empty((batch, heads, n, d), dtype=out_dt) for _ in range(3)]

    def fill(job):
        t, b, h = job
        x = head_normal(seed, t, b, h, n, d, q_gain if t == 0 else 1.0)
        out[t][b, h] = f32_to_bf16_bits(x) if dtype == "bf16" else x   # (numpy rounds to float16 nearest-even)

    jobs = [(t, b, h) for t in range(3) for b in range(batch) for h in range(heads)]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out[0], out[1], out[2]


def make_workload_qkv(w: Workload, q_gain: float = 1.0, threads: int = 8):
    return make_qkv(w.batch, w.heads, w.n_tokens, w.head_dim, w.dtype, w.seed, q_gain, threads)


def sample_rows(seed: int, count: int, batch: int, heads: int, n: int) -> np.ndarray:
    """count seeded-random (batch, head, token row) triples, int64 [count, 3]."""
    rng = np.random.default_rng(seed)
    return np.stack([rng.integers(0, batch, count), rng.integers(0, heads, count),
                     rng.integers(0, n, count)], axis=1).astype(np.int64)
