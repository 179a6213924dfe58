"""Seeded synthetic inputs (gradients, weights, test-only nonzero errors) for the five benchmark workloads.

This module serves both the CPU oracle's tests and the HIP path's tests and benchmark.  It holds none of the
method's arithmetic: it only draws random numbers of a stated distribution into flat fp32 buffers.

The values are zero-centred, like the gradient histograms of the paper's Fig. 1.  A workload's inputs are
fixed by (recipe, seed, torch device type): torch's CPU and GPU generators draw different streams, so a test
generates once, on one device, and hands the same bytes to both sides.

Sub-stream seeds: worker p's gradient at step t uses seed*1_000_003 + t*1_009 + p; the weights use
seed*1_000_003 + 999_983; structure shared by all workers (per-tensor scales) uses seed*1_000_003 + 999_979;
the test-only nonzero error of worker p uses seed*1_000_003 + 500_009 + p.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

from . import shapes

CHUNK = 1 << 24  # elements drawn per call, so temporaries stay at 64 MiB whatever n is


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _chunks(n: int):
    for lo in range(0, n, CHUNK):
        yield lo, min(n, lo + CHUNK)


def _fill_normal(out: torch.Tensor, sigma: float, gen: torch.Generator) -> None:
    for lo, hi in _chunks(out.numel()):
        out[lo:hi].normal_(0.0, sigma, generator=gen)


def _fill_laplace(out: torch.Tensor, b: float, gen: torch.Generator) -> None:
    # Laplace(0, b) = b * Exp(1) * random sign
    for lo, hi in _chunks(out.numel()):
        v = out[lo:hi]
        v.exponential_(1.0, generator=gen)
        sign = torch.randint(0, 2, (hi - lo,), generator=gen, device=out.device, dtype=torch.int8)
        v.mul_(sign.to(torch.float32).mul_(2.0).sub_(1.0)).mul_(b)


def _fill_student_t3(out: torch.Tensor, scale: float, gen: torch.Generator) -> None:
    # t(3) = Z / sqrt(chi2_3 / 3), chi2_3 = sum of three squared standard normals
    for lo, hi in _chunks(out.numel()):
        m = hi - lo
        z = torch.empty(m, device=out.device, dtype=torch.float32).normal_(generator=gen)
        c = torch.zeros(m, device=out.device, dtype=torch.float32)
        t = torch.empty(m, device=out.device, dtype=torch.float32)
        for _ in range(3):
            t.normal_(generator=gen)
            c.addcmul_(t, t)
        c.div_(3.0).sqrt_().clamp_(min=1e-12)
        out[lo:hi] = z.div_(c).mul_(scale)


def _apply_bernoulli(out: torch.Tensor, prob: float, gen: torch.Generator, factor: float) -> None:
    """Multiply each element by `factor` with probability `prob` (factor 0 plants exact zeros)."""
    for lo, hi in _chunks(out.numel()):
        u = torch.rand(hi - lo, generator=gen, device=out.device)
        v = out[lo:hi]
        v.copy_(torch.where(u < prob, v * factor, v))


@dataclass
class Workload:
    name: str
    tensors: shapes.Tensors
    num_workers: int
    seed: int
    recipe: str
    eta: float = 0.1
    steps: int = 1
    params: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return shapes.total(self.tensors)

    # ---- shared structure -------------------------------------------------------------------------
    def tensor_scales(self) -> List[float]:
        """Per-tensor scale, log-uniform in [lo, hi], shared by all workers (drawn on the CPU)."""
        lo, hi = self.params["scale_lo"], self.params["scale_hi"]
        gen = _gen("cpu", self.seed * 1_000_003 + 999_979)
        u = torch.rand(len(self.tensors), generator=gen, dtype=torch.float64)
        return [float(math.exp(math.log(lo) + float(x) * (math.log(hi) - math.log(lo)))) for x in u]

    # ---- per-worker gradient ----------------------------------------------------------------------
    def gradient(self, p: int, step: int = 0, device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n = self.n
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=device)
        assert out.numel() == n and out.dtype == torch.float32
        gen = _gen(out.device, self.seed * 1_000_003 + step * 1_009 + p)
        r = self.recipe
        if r == "normal_zeros":
            _fill_normal(out, self.params["sigma"], gen)
            _apply_bernoulli(out, self.params["zero_prob"], gen, 0.0)
        elif r == "laplace_per_tensor":
            off = 0
            for (_, numel), s in zip(self.tensors, self.tensor_scales()):
                _fill_laplace(out[off:off + numel], s, gen)
                off += numel
        elif r == "lstm_sparse_rows":
            _fill_normal(out, self.params["sigma"], gen)
            rows, cols = self.params["encoder_rows"], self.params["encoder_cols"]
            assert self.tensors[0][1] == rows * cols
            dead = torch.rand(rows, generator=gen, device=out.device) < self.params["zero_row_prob"]
            out[:rows * cols].view(rows, cols)[dead] = 0.0
        elif r == "student_t3":
            _fill_student_t3(out, self.params["scale"], gen)
        elif r == "normal_outliers":
            _fill_normal(out, self.params["sigma"], gen)
            _apply_bernoulli(out, self.params["outlier_prob"], gen, self.params["outlier_factor"])
        else:
            raise ValueError(f"unknown recipe {r!r}")
        return out

    def weights(self, device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty(self.n, dtype=torch.float32, device=device)
        _fill_normal(out, 0.02, _gen(out.device, self.seed * 1_000_003 + 999_983))
        return out

    def initial_error(self, p: int, device="cpu") -> torch.Tensor:
        """Every workload starts from a zero error vector."""
        return torch.zeros(self.n, dtype=torch.float32, device=device)

    def synthetic_error(self, p: int, device="cpu", out: Optional[torch.Tensor] = None,
                        rel_sigma: float = 0.6) -> torch.Tensor:
        """Test-only nonzero error: N(0, (rel_sigma * typical |g|)^2), so that g + e changes sign often.

        Parity tests at full size use it as the `e` input of a single step, because a carried error would
        have to come from one of the two implementations under comparison.
        """
        if out is None:
            out = torch.empty(self.n, dtype=torch.float32, device=device)
        _fill_normal(out, rel_sigma * self.typical_magnitude(), _gen(out.device, self.seed * 1_000_003 + 500_009 + p))
        return out

    def typical_magnitude(self) -> float:
        r = self.recipe
        if r in ("normal_zeros", "lstm_sparse_rows", "normal_outliers"):
            return self.params["sigma"]
        if r == "laplace_per_tensor":
            return math.sqrt(self.params["scale_lo"] * self.params["scale_hi"])
        if r == "student_t3":
            return self.params["scale"]
        raise ValueError(r)


# ---- the five benchmark configurations, and shrunken variants with the same structure ---------------

def config1(n: int = 1_048_576, num_workers: int = 4) -> Workload:
    return Workload("config1_flat", shapes.flat(n), num_workers, seed=0, recipe="normal_zeros", eta=0.1, steps=10,
                    params=dict(sigma=1e-3, zero_prob=0.01))


def config2(width: int = 64, num_classes: int = 1000, num_workers: int = 8) -> Workload:
    return Workload("config2_resnet50", shapes.resnet50(width, num_classes), num_workers, seed=1,
                    recipe="laplace_per_tensor", params=dict(scale_lo=1e-5, scale_hi=1e-2))


def config3(vocab: int = 10000, hidden: int = 1500, num_workers: int = 8) -> Workload:
    return Workload("config3_lstm", shapes.lstm_lm(vocab, hidden), num_workers, seed=2, recipe="lstm_sparse_rows",
                    params=dict(sigma=1e-3, zero_row_prob=0.95, encoder_rows=vocab, encoder_cols=hidden))


def config4(width: int = 64, fc: int = 4096, num_classes: int = 1000, num_workers: int = 16) -> Workload:
    return Workload("config4_vgg16", shapes.vgg16(width, fc, 7, num_classes), num_workers, seed=3,
                    recipe="student_t3", params=dict(scale=1e-4))


def config5(layers: int = 48, d_model: int = 1600, d_ff: int = 6400, vocab: int = 50257,
            truncate_to: Optional[int] = 1_500_000_000, num_workers: int = 4) -> Workload:
    return Workload("config5_transformer", shapes.transformer(layers, d_model, d_ff, vocab, 1024, truncate_to),
                    num_workers, seed=4, recipe="normal_outliers",
                    params=dict(sigma=1e-4, outlier_prob=1e-3, outlier_factor=100.0))


def table1(model: str, num_workers: int = 4) -> Workload:
    """The paper's own small models (Table 1) as per-layer tensor lists, with the per-tensor scales and Laplace
    values of config 2: stand-ins for their gradients, which would need MNIST / CIFAR10 and training."""
    tensors = {"fnn3": shapes.fnn3, "resnet20": shapes.resnet20, "vgg16_cifar": shapes.vgg16_cifar}[model]()
    seed = {"fnn3": 11, "resnet20": 12, "vgg16_cifar": 13}[model]
    return Workload(f"table1_{model}", tensors, num_workers, seed=seed, recipe="laplace_per_tensor",
                    params=dict(scale_lo=1e-5, scale_hi=1e-2))


FULL = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def small(k: int) -> Workload:
    """Same structure and value recipe as config k at a size a CPU oracle finishes in well under a second."""
    if k == 1:
        return config1(n=65_539)
    if k == 2:
        return config2(width=8, num_classes=37)
    if k == 3:
        return config3(vocab=500, hidden=60)
    if k == 4:
        return config4(width=4, fc=96, num_classes=29)
    if k == 5:
        return config5(layers=2, d_model=64, d_ff=256, vocab=997, truncate_to=200_003)
    raise ValueError(k)
