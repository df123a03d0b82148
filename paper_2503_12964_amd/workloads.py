"""Seeded synthetic workloads shaped like the paper's video-latent batches.

This module only draws random numbers and describes shapes.  It holds none of
the method's arithmetic (no rotation, no softmax), so both the GPU tests and
the CPU oracle tests may import it.

Shapes follow the paper's workloads: Table 1 (32 heads x 128 = hidden 4096,
long contexts), Section 3.1 (clips of different shapes packed along the
sequence with micro-batch 1), Section 5.2 (classifier-free guidance gives
batch 2 at inference).  The paper's datasets and weights are not available,
so q, k, v and dout are independent N(0,1) draws rounded to bf16 (unit RMS,
as per-head normalised queries and keys would have).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np

TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "dout": 3, "gain": 4, "dy": 5}


@dataclass(frozen=True)
class Workload:
    name: str
    grids: Tuple[Tuple[int, int, int], ...]   # one latent grid (T, H, W) per packed clip
    n_heads: int
    head_dim: int
    rope_dims: Tuple[int, int, int]           # head_dim split over the t, h, w axes
    seed: int
    backward: bool = True
    theta: float = 10000.0

    @property
    def seqlens(self):
        return [t * h * w for (t, h, w) in self.grids]

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    @property
    def thw(self) -> np.ndarray:
        return np.asarray(self.grids, dtype=np.int32).reshape(-1, 3)

    @property
    def spatial_cu_seqlens(self) -> np.ndarray:
        """Segment boundaries of spatial attention (Section 4.6): every latent frame of every
        clip is its own sequence of H*W tokens.  With t the slowest index of the flatten order
        this is a pure re-reading of the same packed buffer."""
        lens = [h * w for (t, h, w) in self.grids for _ in range(t)]
        return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def pairs(self) -> int:
        """Number of (query, key) pairs per head: sum over clips of N_s**2."""
        return int(sum(n * n for n in self.seqlens))

    def flops(self, backward: bool | None = None, cu_seqlens=None) -> float:
        """Algorithmic flops: 4*D per pair per head forward, 10*D backward.  cu_seqlens
        overrides the clip boundaries (e.g. the spatial view)."""
        bwd = self.backward if backward is None else backward
        per_pair = (4 + (10 if bwd else 0)) * self.head_dim
        pairs = self.pairs if cu_seqlens is None else int(np.sum(np.diff(np.asarray(cu_seqlens, dtype=np.int64)) ** 2))
        return float(per_pair) * self.n_heads * pairs


WORKLOADS = {
    # tiny reference case
    "C1": Workload("C1", ((2, 4, 4),), 2, 64, (16, 24, 24), seed=0),
    # 256px-class latent, batch 2 expressed as two equal segments
    "C2": Workload("C2", ((4, 32, 32), (4, 32, 32)), 16, 128, (32, 48, 48), seed=1),
    # eight clips of different shapes packed together (28,704 tokens)
    "C3": Workload("C3", ((2, 16, 16), (4, 24, 40), (8, 32, 32), (3, 22, 40),
                          (6, 16, 16), (5, 24, 40), (1, 32, 32), (7, 22, 40)),
                   24, 128, (32, 48, 48), seed=2),
    # 720p-class 121-frame latent (headline)
    "C4": Workload("C4", ((16, 44, 80),), 32, 128, (32, 48, 48), seed=3),
    # a 73,728-token context (Table 1) filled with 256-token images (Section 3.1 packs images and videos)
    "P288": Workload("P288", tuple((1, 16, 16) for _ in range(288)), 32, 128, (32, 48, 48), seed=6),
    # one run's worth of the same images (the library launches a call in runs of 256 clips): the shape the
    # short-sequence profile is taken on, so that every kernel has one dispatch per step
    "P256": Workload("P256", tuple((1, 16, 16) for _ in range(256)), 32, 128, (32, 48, 48), seed=7),
    # a long video for temporal attention only (Section 4.6: hundreds of frames): 64 latent frames of the
    # 720p-class grid, 8 heads (bench.py --workload L64-temporal)
    "L64": Workload("L64", ((64, 44, 80),), 8, 128, (32, 48, 48), seed=5),
    # 1080p-class latent, inference denoising step (forward only)
    "C5": Workload("C5", ((16, 68, 120),), 40, 128, (32, 48, 48), seed=4, backward=False),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed: int, tensor: str, shape: Sequence[int], gain: float = 1.0) -> np.ndarray:
    """Independent N(0, gain^2) fp32 draws, reproducible per (seed, tensor name)."""
    rng = np.random.Generator(np.random.Philox(key=[int(seed), TENSOR_IDS[tensor]]))
    x = rng.standard_normal(size=tuple(shape), dtype=np.float32)
    if gain != 1.0:
        x *= np.float32(gain)
    return x


def norm_gain(wl: Workload) -> np.ndarray:
    """Learned gain of the per-head normalisation, fp32 [head_dim]: 1 + 0.25 N(0,1), seeded."""
    return (1.0 + normal_f32(wl.seed, "gain", (wl.head_dim,), 0.25)).astype(np.float32)


def make_inputs(wl: Workload, heads: int | None = None, gain_qk: float = 1.0,
                tensors: Sequence[str] = ("q", "k", "v", "dout")) -> dict:
    """bf16 bit patterns (uint16, [total, heads, head_dim]) for each requested tensor.

    gain_qk > 1 scales q and k to make the softmax peaky (exercises the
    running-max update); the default matches the paper-shaped workloads.
    """
    H = wl.n_heads if heads is None else heads
    shape = (wl.total_tokens, H, wl.head_dim)
    out = {}
    for name in tensors:
        g = gain_qk if name in ("q", "k") else 1.0
        out[name] = f32_to_bf16_bits(normal_f32(wl.seed, name, shape, g))
    return out
