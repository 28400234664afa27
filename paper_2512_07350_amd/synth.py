"""Seeded synthetic inputs for the LP hot path.

Holds shapes, seeds and random draws only -- none of the method's arithmetic.
Both the HIP path (through the binding) and the CPU oracle are fed from here so
that they see identical bits; neither side is imported by this module.

Workload shapes follow the WAN-style latent layout [16, 1 + (F - 1) / 4, H/8, W/8]
with patch (1, 2, 2) (the 480p case is 60 x 104, which is what the paper's
communication table implies for its 49- and 81-frame runs).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

DIM_NAMES = ("T", "H", "W")


@dataclass(frozen=True)
class Workload:
    name: str
    latent: Tuple[int, int, int, int]      # C, T, H, W
    patch: Tuple[int, int, int]            # pT, pH, pW
    K: int
    overlap_patches: int
    dims: Tuple[int, ...]                  # partition dims visited, in order (0=T,1=H,2=W)
    heads: int
    head_dim: int
    layers: int = 1
    overlap_ratio: Optional[float] = None  # r of Sec. 3.3 (O = floor(L r) per dim); overlap_patches is then -1

    def overlap_args(self) -> dict:
        """Keyword arguments of the plan constructors (library and oracle use the same names)."""
        if self.overlap_ratio is not None:
            return {"overlap_patches": -1, "overlap_ratio": float(self.overlap_ratio)}
        return {"overlap_patches": self.overlap_patches}


# The five benchmark configurations (index = position in the baseline's list), then the
# setting of the paper's communication table (49 frames at 480p, K = 4, overlap ratio 0.5 and 1.0)
# and three variations of the 81-frame case.
WORKLOADS = (
    Workload("tiny", (16, 5, 16, 16), (1, 2, 2), 2, 1, (2,), 4, 64),
    Workload("wan1.3b-33f-480p", (16, 9, 60, 104), (1, 2, 2), 4, 1, (0, 1, 2), 12, 128),
    Workload("wan1.3b-81f-480p", (16, 21, 60, 104), (1, 2, 2), 4, 2, (1,), 12, 128),
    Workload("dit14b-81f-720p", (16, 21, 90, 160), (1, 2, 2), 8, 2, (2,), 40, 128),
    Workload("wan1.3b-81f-480p-loop", (16, 21, 60, 104), (1, 2, 2), 4, 2, (0, 1, 2), 12, 128, layers=30),
    Workload("wan1.3b-49f-480p-r0.5", (16, 13, 60, 104), (1, 2, 2), 4, -1, (0, 1, 2), 12, 128, overlap_ratio=0.5),
    Workload("wan1.3b-49f-480p-r1.0", (16, 13, 60, 104), (1, 2, 2), 4, -1, (0, 1, 2), 12, 128, overlap_ratio=1.0),
    # the paper's sweeps over the number of devices and its temporal-only ablation, at 81 frames
    Workload("wan1.3b-81f-480p-K2", (16, 21, 60, 104), (1, 2, 2), 2, 2, (0, 1, 2), 12, 128),
    Workload("wan1.3b-81f-480p-K8", (16, 21, 60, 104), (1, 2, 2), 8, 2, (0, 1, 2), 12, 128),
    Workload("wan1.3b-81f-480p-temporal-only", (16, 21, 60, 104), (1, 2, 2), 4, 2, (0,), 12, 128),
    # the longest clip of the paper's duration sweep: 10 s at 16 frames per second = 161 frames = 41 latent frames
    Workload("wan1.3b-161f-480p-r0.5", (16, 41, 60, 104), (1, 2, 2), 4, -1, (0, 1, 2), 12, 128, overlap_ratio=0.5),
)


def seed_for(cfg: int, dim: int, k: int, tensor: int = 0) -> int:
    """One stream per (config, partition dim, partition, tensor id)."""
    return 0x4C500000 + 0x1000 * tensor + 0x100 * cfg + 0x10 * dim + k


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to binary32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed: int, shape: Sequence[int], substream: int = 0) -> np.ndarray:
    """N(0,1) binary32 tensor from a fixed stream.  `substream` selects one of the disjoint
    stretches of that seed's Philox sequence (each 2^128 draws long), so tensors that share a
    seed never share values, whatever other seeds are in use."""
    bits = np.random.Philox(seed)
    if substream:
        bits = bits.jumped(substream)
    return np.random.Generator(bits).standard_normal(size=tuple(shape), dtype=np.float32)


def latent(seed: int, shape: Sequence[int]) -> np.ndarray:
    return normal_f32(seed, shape)


def index_coded(shape: Sequence[int]) -> np.ndarray:
    """Latent whose value at linear index i is float(i mod 2^20): any mis-indexing shows."""
    n = int(np.prod(shape))
    return (np.arange(n, dtype=np.int64) % (1 << 20)).astype(np.float32).reshape(tuple(shape))


def qkv_bf16(seed: int, n_tokens: int, heads: int, head_dim: int):
    """Q, K, V ~ N(0,1) rounded to bf16, each uint16 [n_tokens, heads, head_dim]."""
    out = []
    for t in range(3):
        x = normal_f32(seed, (n_tokens, heads, head_dim), substream=t + 1)
        out.append(f32_to_bf16_bits(x))
    return tuple(out)


def sample_rows(n: int, count: int, seed: int, tile: int = 64) -> np.ndarray:
    """Query rows for sampled checks: first, last, the rows on both sides of every tile edge
    among the first four and the last four tiles, then seeded random rows up to `count`;
    sorted, unique."""
    picks = {0, n - 1}
    last_edge = (n // tile) * tile
    edges = [m * tile for m in range(1, 5)] + [last_edge - m * tile for m in range(0, 4)]
    for edge in edges:
        for r in (edge - 1, edge, edge + 1):
            if 0 <= r < n:
                picks.add(r)
    rng = np.random.Generator(np.random.Philox(seed))
    while len(picks) < min(count, n):
        picks.add(int(rng.integers(0, n)))
    return np.array(sorted(picks), dtype=np.int64)
