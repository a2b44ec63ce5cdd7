"""Seeded synthetic gradient sets shaped like the paper's two ImageNet models.

This module only describes tensor shapes and draws random numbers.  It holds
none of the method's arithmetic (no layout, bucketing, casting, scoring,
selection or reduction), so both the HIP path and the CPU checker may be fed
from it.

The paper trains AlexNet and ResNet-50 on ImageNet-1K (Section 2.3, the figure
listing per-layer parameter counts); those gradients are not available, so
tensors of the same shapes filled with seeded normal noise stand in for them:
for worker p and tensor l the standard deviation sigma[l, p] is drawn once,
log-uniform in [1e-4, 1e-1], and every iteration t draws fresh N(0, sigma^2)
values from a generator seeded by (seed, t, p, l).

Tensor lists are in ID order 1..m = forward order of the network (weight before
bias; conv weight, BN gamma, BN beta; the downsample branch after conv3; the
classifier last).  Backward produces them in the opposite order.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch


def tiny_sizes() -> List[int]:
    return [4096, 16384, 65536, 131072, 262144, 524288]


def alexnet_sizes() -> List[int]:
    """Grouped two-tower AlexNet: 16 tensors, 60 965 224 parameters."""
    convs = [(96, 3, 11, 11), (256, 48, 5, 5), (384, 256, 3, 3),
             (384, 192, 3, 3), (256, 192, 3, 3)]
    fcs = [(4096, 9216), (4096, 4096), (1000, 4096)]
    out: List[int] = []
    for s in convs:
        out += [int(np.prod(s)), s[0]]
    for s in fcs:
        out += [s[0] * s[1], s[0]]
    return out


def resnet50_sizes() -> List[int]:
    """ResNet-50 (bottleneck stages [3,4,6,3]): 161 tensors, 25 557 032 parameters."""
    out: List[int] = [64 * 3 * 7 * 7, 64, 64]
    inplanes = 64
    for width, blocks in zip((64, 128, 256, 512), (3, 4, 6, 3)):
        for b in range(blocks):
            out += [width * inplanes, width, width]            # 1x1 reduce + BN
            out += [width * width * 9, width, width]           # 3x3 + BN
            out += [4 * width * width, 4 * width, 4 * width]   # 1x1 expand + BN
            if b == 0:                                         # projection shortcut
                out += [4 * width * inplanes, 4 * width, 4 * width]
            inplanes = 4 * width
    out += [1000 * 2048, 1000]
    return out


@dataclass
class Workload:
    """One benchmark / parity configuration (shapes and scalars only)."""
    name: str
    sizes: List[int]               # tensor element counts, ID order 1..m
    P: int                         # simulated workers
    chunk: int                     # chunk elements, 0 = dense path
    density: float                 # fraction of chunks selected (CSC only)
    loss_scale: float
    theta: int                     # fusion threshold in wire elements
    iterations: int = 1
    mu: float = 1.0
    seed: int = 1902_06855
    wire: str = "f16"
    extra: dict = field(default_factory=dict)
    grad: str = "f32"              # element type the gradients arrive in

    @property
    def m(self) -> int:
        return len(self.sizes)

    @property
    def N(self) -> int:
        return int(sum(self.sizes))

    def k_for(self, n_chunks: int) -> int:
        """Selected-chunk count for this density: ceil(density * n_chunks) in [1, n_chunks]."""
        return max(1, min(n_chunks, math.ceil(self.density * n_chunks - 1e-9)))


MB = 1 << 20


def config(name: str) -> Workload:
    """The configurations this build is measured and checked on, and the rungs
    below them of the ladder of Tables 1-2 (one allreduce per tensor in fp32,
    the same in fp16, then lazy allreduce, then sparse communication), plus the
    fp16-resident pool of Section 3.1 reduced in place."""
    if name == "tiny":
        return Workload("tiny", tiny_sizes(), P=4, chunk=4096, density=0.25,
                        loss_scale=1024.0, theta=1 << 40)
    if name == "alexnet_dense":
        return Workload("alexnet_dense", alexnet_sizes(), P=8, chunk=0, density=1.0,
                        loss_scale=1024.0, theta=32 * MB // 2)
    if name == "resnet50_dense_4mb":
        return Workload("resnet50_dense_4mb", resnet50_sizes(), P=8, chunk=0, density=1.0,
                        loss_scale=128.0, theta=4 * MB // 2)
    if name == "resnet50_dense_64mb":
        return Workload("resnet50_dense_64mb", resnet50_sizes(), P=8, chunk=0, density=1.0,
                        loss_scale=128.0, theta=64 * MB // 2)
    if name == "alexnet_csc":
        return Workload("alexnet_csc", alexnet_sizes(), P=16, chunk=32768, density=0.10,
                        loss_scale=1024.0, theta=1 << 40, iterations=10)
    if name == "resnet50_csc":
        return Workload("resnet50_csc", resnet50_sizes(), P=64, chunk=8192, density=0.01,
                        loss_scale=128.0, theta=1 << 40, iterations=20)
    base = {"alexnet": (alexnet_sizes, 1024.0), "resnet50": (resnet50_sizes, 128.0)}
    for net, (sizes, S) in base.items():
        if name == net + "_pertensor_fp32":    # baseline: every tensor its own fp32 allreduce
            return Workload(name, sizes(), P=8, chunk=0, density=1.0, loss_scale=1.0, theta=0, wire="f32")
        if name == net + "_pertensor_fp16":    # + mixed precision
            return Workload(name, sizes(), P=8, chunk=0, density=1.0, loss_scale=S, theta=0)
        if name == net + "_fp16pool":          # fp16 gradients already in the pool, reduced in place
            return Workload(name, sizes(), P=8, chunk=0, density=1.0, loss_scale=S, theta=32 * MB // 2,
                            grad="f16", extra={"zero_copy": True})
    if name == "alexnet_csc_hier":             # 16 ranks in 4 groups: the example of Section 2.4's figure
        w = config("alexnet_csc")
        w.name, w.extra = name, {"groups": 4}
        return w
    if name == "resnet50_csc_hier":            # 64 ranks in 8 groups of 8
        w = config("resnet50_csc")
        w.name, w.extra = name, {"groups": 8}
        return w
    if name == "alexnet_dense_hier":           # 8 ranks in 2 groups
        w = config("alexnet_dense")
        w.name, w.extra = name, {"groups": 2}
        return w
    if name.endswith("_p1") and name[:-3] in ("alexnet_csc", "resnet50_csc"):
        # one worker: the shape each GPU of a real job runs (its own gradients, its own historical
        # gradient; the exchange itself is the network's and degenerates to a copy here)
        w = config(name[:-3])
        w.name, w.P = name, 1
        return w
    for c in (2048, 4096):                     # the ResNet-50 set cut into short chunks
        if name == f"resnet50_csc_c{c}":
            w = config("resnet50_csc")
            w.name, w.chunk, w.P = name, c, 16
            return w
    if name == "alexnet_csc_fp16in":           # sparse path fed with fp16 gradients
        w = config("alexnet_csc")
        w.name, w.grad = name, "f16"
        return w
    raise KeyError(name)


LADDER_NAMES = ("alexnet_pertensor_fp32", "alexnet_pertensor_fp16", "alexnet_fp16pool", "alexnet_csc_fp16in",
                "resnet50_pertensor_fp32", "resnet50_pertensor_fp16", "resnet50_fp16pool",
                "alexnet_dense_hier", "alexnet_csc_hier", "resnet50_csc_hier",
                "resnet50_csc_c4096", "resnet50_csc_c2048")

CONFIG_NAMES = ("tiny", "alexnet_dense", "resnet50_dense_4mb", "resnet50_dense_64mb",
                "alexnet_csc", "resnet50_csc")


def scaled(w: Workload, divisor: int, name: Optional[str] = None) -> Workload:
    """A copy of `w` whose tensors are `divisor` times smaller (each at least 8,
    rounded to a multiple of 8) with chunk and theta shrunk alike; keeps the
    tensor count and the size mix."""
    sizes = [max(8, (s // divisor) // 8 * 8) for s in w.sizes]
    chunk = 0 if w.chunk == 0 else max(64, w.chunk // divisor)
    theta = w.theta if w.theta >= (1 << 40) else max(1, w.theta // divisor)
    return Workload(name or f"{w.name}_div{divisor}", sizes, w.P, chunk, w.density,
                    w.loss_scale, theta, w.iterations, w.mu, w.seed, w.wire, dict(w.extra), w.grad)


def _mix(*vals: int) -> int:
    """Deterministic 63-bit hash of a tuple of small integers (splitmix-style)."""
    x = 0x9E3779B97F4A7C15
    for v in vals:
        x ^= (int(v) + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
        x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 29
    return x & 0x7FFFFFFFFFFFFFFF


def stream_seed(*vals: int) -> int:
    """Seed of an independent random stream named by a tuple of small integers."""
    return _mix(*vals)


def sigma_table(w: Workload) -> np.ndarray:
    """sigma[l, p], log-uniform in [1e-4, 1e-1], fixed for the whole run."""
    rng = np.random.default_rng(_mix(w.seed, 0xA11CE))
    e = rng.uniform(-4.0, -1.0, size=(w.m, w.P))
    return (10.0 ** e).astype(np.float32)


def gradient_tensor(w: Workload, sig: np.ndarray, t: int, p: int, l: int,
                    device: str = "cpu") -> torch.Tensor:
    """Tensor l (0-based ID-order index) of worker p at iteration t, fp32 (or
    those values converted to fp16 when the workload's gradients arrive so)."""
    g = torch.Generator(device=device)
    g.manual_seed(_mix(w.seed, t, p, l))
    x = torch.randn(w.sizes[l], generator=g, device=device, dtype=torch.float32)
    x.mul_(float(sig[l, p]))
    return x.to(torch.float16) if w.grad == "f16" else x


def gradients(w: Workload, t: int, device: str = "cpu",
              sig: Optional[np.ndarray] = None) -> List[List[torch.Tensor]]:
    """grads[p][l]: separately allocated tensors, ID order, for iteration t.

    The values depend on `device` (torch's CPU and GPU generators differ); a
    caller that needs the same bits on both sides generates once and copies.
    """
    if sig is None:
        sig = sigma_table(w)
    return [[gradient_tensor(w, sig, t, p, l, device) for l in range(w.m)]
            for p in range(w.P)]


def integer_gradients(sizes: Sequence[int], P: int, seed: int, lo: int = -8, hi: int = 8
                      ) -> List[List[torch.Tensor]]:
    """Small-integer-valued fp32 tensors: every partial sum is exactly
    representable, which makes sums independent of their order."""
    out = []
    for p in range(P):
        row = []
        for l, n in enumerate(sizes):
            g = torch.Generator()
            g.manual_seed(_mix(seed, p, l, 77))
            row.append(torch.randint(lo, hi + 1, (n,), generator=g).to(torch.float32))
        out.append(row)
    return out
