"""Seeded synthetic gradient workloads.

This module only manufactures INPUTS (gradient vectors and an initial
threshold); it holds none of the sparsifier's arithmetic and is the one piece
that both the GPU library's callers and the CPU oracle's tests draw from.  A
gradient is generated once (on whatever device is asked for) and the same
bytes are handed to both sides.

The five workloads stand in for the gradient tensors of the networks the
paper trains (its datasets and trained weights are not available): the sizes
are those of public architectures, the values are random with heavy tails,
per-layer scale spread, scale drift over iterations, or a skewed head, so that
threshold scaling and partition rebalancing have something to track.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # 1-based position in the list of configurations
    n_g: int              # number of gradients
    block_size: int       # b
    n_parts: int          # P
    density: float        # d
    iters: int            # iterations of the full trajectory
    seed: int
    kind: str             # laplace | seg_laplace | seg_student | drift_laplace | skew_laplace
    n_segments: int = 0
    scale: float = 1e-3

    @property
    def n_blocks(self) -> int:
        return -(-self.n_g // self.block_size)

    def scaled(self, n_g: int, block_size: Optional[int] = None, n_parts: Optional[int] = None,
               iters: Optional[int] = None) -> "Workload":
        """Same value recipe at a smaller size (for tests the oracle finishes in seconds)."""
        return replace(self, n_g=n_g, block_size=block_size or self.block_size,
                       n_parts=n_parts or self.n_parts, iters=iters or self.iters,
                       name=f"{self.name}@{n_g}")


WORKLOADS = {
    1: Workload("cfg1-iid-laplace-1M", 1, 1_048_576, 256, 4, 0.01, 20, 0, "laplace"),
    2: Workload("cfg2-resnet18-size-62seg", 2, 11_689_512, 4096, 8, 0.001, 100, 1, "seg_laplace",
                n_segments=62),
    3: Workload("cfg3-resnet50-size-161seg-student", 3, 25_557_032, 4096, 16, 0.01, 100, 2,
                "seg_student", n_segments=161),
    4: Workload("cfg4-vgg16-size-drift", 4, 138_357_544, 16384, 32, 0.001, 200, 3, "drift_laplace"),
    5: Workload("cfg5-transformer-size-skew", 5, 1_500_000_000, 65536, 64, 0.0001, 50, 4,
                "skew_laplace"),
}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _laplace_(out: torch.Tensor, gen: torch.Generator) -> torch.Tensor:
    """Fill `out` with unit-scale Laplace draws (inverse CDF of a symmetric uniform)."""
    chunk = 1 << 27
    for s in range(0, out.numel(), chunk):
        o = out[s:s + chunk]
        o.uniform_(-1.0, 1.0, generator=gen)
        mag = o.abs().clamp_(max=1.0 - 2.0 ** -24)
        mag.neg_().log1p_().neg_()
        o.copy_(torch.where(o < 0, -mag, mag))
    return out


def _segments(w: Workload, lo_exp: float, hi_exp: float):
    """Contiguous segment sizes (log-uniform weights) and per-segment scales (log-uniform)."""
    gen = _gen("cpu", 7919 * (w.seed + 1))
    u = torch.rand(w.n_segments, generator=gen, dtype=torch.float64)
    weights = 10.0 ** (2.0 + 4.5 * u)
    sizes = torch.floor(weights / weights.sum() * w.n_g).to(torch.int64).clamp_(min=1)
    sizes[-1] += w.n_g - int(sizes.sum())
    if sizes[-1] < 1:  # only reachable for tiny scaled-down n_g
        sizes = torch.full((w.n_segments,), w.n_g // w.n_segments, dtype=torch.int64)
        sizes[-1] += w.n_g - int(sizes.sum())
    v = torch.rand(w.n_segments, generator=gen, dtype=torch.float64)
    scales = 10.0 ** (lo_exp + (hi_exp - lo_exp) * v)
    return sizes, scales


class GradientSource:
    """Produces the gradient of iteration `step` of a workload on a device."""

    def __init__(self, w: Workload, device="cpu"):
        self.w = w
        self.device = torch.device(device)
        self._scale_vec = None
        if w.kind in ("seg_laplace", "seg_student"):
            lo, hi = (-5.0, -2.0) if w.kind == "seg_laplace" else (-4.0, -1.0)
            sizes, scales = _segments(w, lo, hi)
            self.segment_sizes, self.segment_scales = sizes, scales
            self._scale_vec = torch.repeat_interleave(
                scales.to(torch.float32), sizes).to(self.device)

    def grad(self, step: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        w = self.w
        if out is None:
            out = torch.empty(w.n_g, dtype=torch.float32, device=self.device)
        gen = _gen(self.device, (w.seed + 1) * 1_000_003 + step)
        if w.kind == "laplace":
            _laplace_(out, gen).mul_(w.scale)
        elif w.kind == "seg_laplace":
            _laplace_(out, gen).mul_(self._scale_vec)
        elif w.kind == "seg_student":
            z = torch.empty(w.n_g, dtype=torch.float32, device=self.device)
            den = torch.zeros(w.n_g, dtype=torch.float32, device=self.device)
            for _ in range(3):
                z.normal_(generator=gen)
                den.addcmul_(z, z)
            den.div_(3.0).sqrt_().clamp_(min=1e-20)
            out.normal_(generator=gen)
            out.div_(den).mul_(self._scale_vec).mul_(1e-3)
        elif w.kind == "drift_laplace":
            last = max(w.iters - 1, 1)
            s_t = 1e-2 * (1e-2) ** (min(step, last) / last)
            _laplace_(out, gen).mul_(s_t)
        elif w.kind == "skew_laplace":
            _laplace_(out, gen).mul_(w.scale)
            out[: w.n_g // 20].mul_(20.0)
        else:
            raise ValueError(w.kind)
        return out


def initial_threshold(g0: torch.Tensor, density: float) -> float:
    """The |x| order statistic at 1-d of a 1-in-100 sample of the first gradient."""
    sample = g0[::100].abs().to(torch.float32)
    m = sample.numel()
    rank = max(int(math.ceil((1.0 - density) * m)) - 1, 0)
    srt, _ = torch.sort(sample)
    thr = float(srt[min(rank, m - 1)])
    if not thr > 0.0:
        pos = srt[srt > 0]
        thr = float(pos[0]) if pos.numel() else 1e-30
    return thr
