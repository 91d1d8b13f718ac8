"""Seeded synthetic inputs shaped like the paper's workloads.

The paper trains ImageNet / CIFAR / AN4 networks (Sec. 5, Table 1); neither the
datasets nor trained weights are needed for the Encode / Decode kernels, so the
gradients here are synthetic stand-ins with the parameter counts of Table 1
(ResNet50 25M, VGG19 143M, LSTM 13M) laid out as a flat concatenation of
tensors, each tensor with its own scale, and the bucket / bit settings the
experiments report (Sec. 5: bucket 512 with 4 and 8 bits, 8192 with 4 bits).

This module only draws random numbers; it contains none of the method's
arithmetic and is shared by the tests, the benchmark and the oracle's callers.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace

import torch

CODE_SPARSE, CODE_DENSE, CODE_FIXED = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    s: int
    d: int            # bucket size; d >= n means one bucket
    code: int
    K: int            # peers whose messages are decoded and summed
    eta: float
    dist: str         # normal | laplace_lognormal | normal_loguniform | student_t | normal_outliers
    tensors: tuple = field(default_factory=tuple)  # sizes of the concatenated tensors
    seed: int = 0     # Philox seed of the quantizer
    note: str = ""


def _geometric_sizes(count: int, lo: float, hi: float) -> list:
    r = (hi / lo) ** (1.0 / (count - 1))
    return [int(round(lo * r ** i)) for i in range(count)]


def _c2_tensors(n: int = 25_600_000) -> tuple:
    raw = _geometric_sizes(161, 1_000, 2_400_000)
    scale = n / sum(raw)
    sizes = [max(1, int(x * scale)) for x in raw]
    sizes[-1] += n - sum(sizes)
    return tuple(sizes)


def _c3_tensors(n: int = 143_000_000) -> tuple:
    small = _geometric_sizes(16, 1_700, 2_400_000)
    sizes = small + [16_800_000, 4_100_000]
    sizes.append(n - sum(sizes))
    return tuple(sizes)


C1 = Workload("c1", 1 << 20, 4, 512, CODE_SPARSE, 2, 0.1, "normal", (1 << 20,),
              note="2-bit levels, bucket 512, Elias-coded; N(0, 1e-3^2)")
C2 = Workload("c2", 25_600_000, 16, 512, CODE_SPARSE, 8, 0.1, "laplace_lognormal", _c2_tensors(),
              note="ResNet50-sized: 161 tensors, per-tensor log-normal scale x Laplace")
C3 = Workload("c3", 143_000_000, 256, 512, CODE_FIXED, 16, 0.1, "normal_loguniform",
              _c3_tensors(), note="VGG19-sized: 19 tensors, fixed-width 8-bit level + sign")
C4 = Workload("c4", 13_000_000, 1, 13_000_000, CODE_SPARSE, 16, 0.1, "student_t",
              (3_000_000,) * 4 + (1_000_000,),
              note="LSTM-sized sparse regime: s=1, one bucket of n, Student-t(3) x 1e-3")
C5 = Workload("c5", 1_000_000_000, 4, 8192, CODE_SPARSE, 16, 0.1, "normal_outliers",
              (1_000_000_000,), note="stress: N(0, 1e-3^2), 0.1% entries x100, bucket 8192")

WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def scaled(w: Workload, n: int) -> Workload:
    """The same workload shrunk to n elements (tensor sizes in proportion)."""
    if n >= w.n:
        return w
    f = n / w.n
    sizes = [max(1, int(t * f)) for t in w.tensors]
    sizes[-1] += n - sum(sizes)
    if sizes[-1] < 1:  # rounding pushed the small tensors over: trim from the largest
        sizes = [n]
    d = n if w.d >= w.n else w.d
    return replace(w, name=f"{w.name}@{n}", n=n, d=d, tensors=tuple(sizes))


def _generator(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def gradient(w: Workload, k: int, device="cpu", base_seed: int = 1234) -> torch.Tensor:
    """Peer k's fp32 gradient for workload w, on `device` (n floats)."""
    dev = torch.device(device)
    gen = _generator(dev, base_seed + 7919 * k)
    # per-tensor scales are drawn on the CPU so that they do not depend on the device
    cg = _generator("cpu", base_seed * 31 + k)
    out = torch.empty(w.n, dtype=torch.float32, device=dev)
    off = 0
    for size in w.tensors:
        seg = out[off:off + size]
        if w.dist == "normal":
            seg.normal_(0.0, 1e-3, generator=gen)
        elif w.dist == "laplace_lognormal":
            scale = math.exp(float(torch.randn((), generator=cg)) * 1.5 - 7.0)
            # inverse CDF of Laplace(0, 1); the draw is kept off 0 so the log stays finite
            u = torch.rand(size, generator=gen, device=dev).clamp_(1e-7, 1.0 - 1e-7) - 0.5
            seg.copy_(-scale * torch.sign(u) * torch.log1p(-2.0 * u.abs()))
        elif w.dist == "normal_loguniform":
            e = float(torch.rand((), generator=cg)) * 3.0 - 5.0  # sigma in [1e-5, 1e-2]
            seg.normal_(0.0, 10.0 ** e, generator=gen)
        elif w.dist == "student_t":
            chunk = 1 << 22
            for c0 in range(0, size, chunk):
                c1 = min(size, c0 + chunk)
                z = torch.randn(c1 - c0, generator=gen, device=dev)
                chi = torch.randn(3, c1 - c0, generator=gen, device=dev).square().sum(0) / 3.0
                seg[c0:c1] = 1e-3 * z / chi.sqrt()
        elif w.dist == "normal_outliers":
            chunk = 1 << 26
            for c0 in range(0, size, chunk):
                c1 = min(size, c0 + chunk)
                part = seg[c0:c1]
                part.normal_(0.0, 1e-3, generator=gen)
                hit = torch.rand(c1 - c0, generator=gen, device=dev) < 1e-3
                part.mul_(torch.where(hit, 100.0, 1.0))
        else:
            raise ValueError(w.dist)
        off += size
    assert off == w.n
    return out


def parameters(w: Workload, device="cpu", base_seed: int = 1234) -> torch.Tensor:
    """The model vector x ~ U(-1, 1)."""
    dev = torch.device(device)
    gen = _generator(dev, base_seed + 1_000_003)
    x = torch.empty(w.n, dtype=torch.float32, device=dev)
    chunk = 1 << 26
    for c0 in range(0, w.n, chunk):
        c1 = min(w.n, c0 + chunk)
        x[c0:c1].uniform_(-1.0, 1.0, generator=gen)
    return x
