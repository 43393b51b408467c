"""Seeded synthetic inputs for the Slim-DP communication-set path.

This module holds NO arithmetic of the method: it only draws weights and per-worker
updates with the shapes, sizes and value distributions of the five benchmark
configurations, and derives the integer set sizes from the percentages.  The same
arrays are handed bit-for-bit to the HIP library and to the CPU oracle.

The paper trains VGG-16 ("about 140M" parameters) and GoogLeNet on ImageNet with 4 or 8
workers (section 4.1); neither the data nor the trained weights are available here, so
Gaussian / Laplace vectors of the same length stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

WEIGHT_SEED = 1
EXPLORE_SEED = 0


def gradient_seed(iteration: int, worker: int) -> int:
    return 1000 * iteration + worker + 1


def round_through_fp16(a: np.ndarray) -> np.ndarray:
    """binary32 -> binary16 (round to nearest even) -> binary32.  torch's cast is the same IEEE
    conversion as NumPy's and many times faster on 1e8 elements; either gives the same bits."""
    try:
        import torch
        return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float16).to(torch.float32).numpy()
    except ImportError:
        return a.astype(np.float16).astype(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    W: int
    weight_dist: str            # "normal" | "laplace_fp16" | "fan_in"
    weight_scale: float
    grad_sigma: float
    grad_fp16: bool = False
    core_pct: int = 10          # core = floor(n_s * core_pct / 100) per segment
    explore_pct: int = 2        # explorer = floor((n_s - k_s) * explore_pct / 100) per segment
    c: float = 1.0
    lr: float = 0.01
    n_seg: int = 1
    iterations: int = 1
    reselect_every: int = 1
    seg_off: Optional[tuple] = field(default=None)

    # ---- segment table -------------------------------------------------------------
    def segment_offsets(self) -> np.ndarray:
        if self.seg_off is not None:
            return np.asarray(self.seg_off, dtype=np.uint64)
        if self.n_seg == 1:
            return np.array([0, self.n], dtype=np.uint64)
        # sizes log-uniform in [1e3, 1e6], rescaled to the total; the remainder after the
        # floor goes one element each to the first segments
        rng = np.random.Generator(np.random.PCG64(WEIGHT_SEED + 7919))
        raw = np.exp(rng.uniform(np.log(1e3), np.log(1e6), size=self.n_seg))
        sizes = np.floor(raw * (self.n / raw.sum())).astype(np.int64)
        sizes = np.maximum(sizes, 1)
        rem = self.n - int(sizes.sum())
        j = 0
        while rem != 0:
            step = 1 if rem > 0 else -1
            if sizes[j % self.n_seg] + step >= 1:
                sizes[j % self.n_seg] += step
                rem -= step
            j += 1
        off = np.zeros(self.n_seg + 1, dtype=np.uint64)
        off[1:] = np.cumsum(sizes).astype(np.uint64)
        assert int(off[-1]) == self.n
        return off

    def k_seg(self) -> np.ndarray:
        off = self.segment_offsets().astype(np.int64)
        sizes = off[1:] - off[:-1]
        return (sizes * self.core_pct // 100).astype(np.uint64)

    def m_seg(self) -> np.ndarray:
        off = self.segment_offsets().astype(np.int64)
        sizes = off[1:] - off[:-1]
        k = sizes * self.core_pct // 100
        return ((sizes - k) * self.explore_pct // 100).astype(np.uint64)

    @property
    def k(self) -> int:
        return int(self.k_seg().sum())

    @property
    def m(self) -> int:
        return int(self.m_seg().sum())

    # ---- arrays ---------------------------------------------------------------------
    def weights(self) -> np.ndarray:
        rng = np.random.Generator(np.random.PCG64(WEIGHT_SEED))
        if self.weight_dist == "normal":
            w = rng.standard_normal(self.n, dtype=np.float32)
            w *= np.float32(self.weight_scale)
            return w
        if self.weight_dist == "laplace_fp16":
            w = rng.laplace(0.0, self.weight_scale, size=self.n).astype(np.float32)
            return round_through_fp16(w)
        if self.weight_dist == "fan_in":
            # per segment: variance 2 / fan_in with fan_in = segment size / 64
            off = self.segment_offsets().astype(np.int64)
            w = rng.standard_normal(self.n, dtype=np.float32)
            for s in range(len(off) - 1):
                fan_in = max(1.0, (off[s + 1] - off[s]) / 64.0)
                w[off[s]:off[s + 1]] *= np.float32(np.sqrt(2.0 / fan_in))
            return w
        raise ValueError(self.weight_dist)

    def gradient(self, iteration: int, worker: int) -> np.ndarray:
        rng = np.random.Generator(np.random.PCG64(gradient_seed(iteration, worker)))
        g = rng.standard_normal(self.n, dtype=np.float32)
        g *= np.float32(self.grad_sigma)
        if self.grad_fp16:
            g = round_through_fp16(g)
        return g

    def gradients(self, iteration: int = 0) -> List[np.ndarray]:
        return [self.gradient(iteration, k) for k in range(self.W)]

    def scaled(self, n: int, **kw) -> "Workload":
        """Same recipe at another length (parity-test sizes the oracle finishes in seconds)."""
        params = dict(n=int(n), name=f"{self.name}@{n}", seg_off=None)
        params.update(kw)
        return replace(self, **params)


TINY = Workload("tiny", 1_000_000, 4, "normal", 0.05, 1e-3)
GOOGLENET = Workload("googlenet_seg57", 6_998_552, 4, "fan_in", 0.0, 1e-3, n_seg=57)
VGG16 = Workload("vgg16_flat", 138_357_544, 8, "normal", 0.01, 1e-4)
STRESS = Workload("tie_stress", 138_357_544, 16, "laplace_fp16", 0.01, 1e-4, grad_fp16=True,
                  core_pct=5, explore_pct=1)
LOOP = Workload("vgg16_loop20", 138_357_544, 8, "normal", 0.01, 1e-4, iterations=20,
                reselect_every=5)

CONFIGS = [TINY, GOOGLENET, VGG16, STRESS, LOOP]
BY_NAME = {c.name: c for c in CONFIGS}
