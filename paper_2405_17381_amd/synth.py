"""Seeded synthetic workloads for causal linear attention with decay.

This module only draws random tensors and decay rates; it holds none of the
method's arithmetic, so both the CPU oracle's tests and the HIP path's tests
can take their inputs from it without sharing any computation.

Every tensor is `[B, H, n, d]`, contiguous, generated on the host in fp32 with
`torch.Generator(device="cpu").manual_seed(seed)` in the fixed order Q, K, V, dO.
The 1/sqrt(d) factor is baked into Q, K, V because the method itself applies
no scaling (Sec. 3.1 drops softmax and scaling).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20240517


def lambda_geometric(lo: float, hi: float, count: int) -> List[float]:
    """`count` decay rates spaced geometrically from `lo` to `hi` inclusive."""
    if count == 1:
        return [float(lo)]
    return [float(lo * (hi / lo) ** (i / (count - 1))) for i in range(count)]


def lambda_exp_schedule(H: int) -> List[float]:
    """lambda_h = exp(-(8/H) * (h+1) / 8) = exp(-(h+1)/H), h = 0..H-1
    (a per-head exponential schedule in the spirit of Sec. 4.1's decay rule)."""
    return [float(math.exp(-(h + 1) / H)) for h in range(H)]


@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16"
    B: int
    H: int
    n: int
    d: int
    lambdas: List[float]
    seed: int
    silu_qk: bool = False           # Q, K = silu(N(0,1)) / sqrt(d)
    note: str = ""

    def __post_init__(self):
        # The C ABI takes the decay rates as float32: hold exactly those values, so that the
        # library and the oracle are given the same numbers (like tensor values after their cast).
        self.lambdas = [float(np.float32(x)) for x in self.lambdas]

    @property
    def tokens(self) -> int:
        return self.B * self.n


def _c3_points() -> List[Tuple[int, int]]:
    return [(32, 2048), (16, 4096), (8, 8192), (4, 16384), (2, 32768), (1, 65536)]


def workload(name: str) -> Workload:
    """Named workloads.

    c1            fp32, B=1 H=2 n=256 d=64, lambda=(1.0, 0.99)
    c2            bf16, B=4 H=16 n=2048 d=64, lambda_h = exp(-(h+1)/H)
    c3_<n>        bf16 sweep point, H=16 d=128, B*n = 65536, n in 2048..65536,
                  lambda_h geometric in [0.9, 0.9999]
    c4            bf16, B=8 H=32 n=4096 d=128, Q,K through SiLU, lambda geometric
    c5            bf16, B=1 H=32 n=131072 d=128, heads 0..15 lambda=1, heads
                  16..31 geometric in [0.95, 0.9999]
    """
    if name == "c1":
        return Workload("c1", "f32", 1, 2, 256, 64, [1.0, 0.99], BASE_SEED + 1)
    if name == "c2":
        return Workload("c2", "bf16", 4, 16, 2048, 64, lambda_exp_schedule(16), BASE_SEED + 2)
    if name.startswith("c3_"):
        n = int(name[3:])
        for (B, nn) in _c3_points():
            if nn == n:
                return Workload(name, "bf16", B, 16, n, 128,
                                lambda_geometric(0.9, 0.9999, 16), BASE_SEED + 3)
        raise KeyError(name)
    if name == "c4":
        return Workload("c4", "bf16", 8, 32, 4096, 128,
                        lambda_geometric(0.9, 0.9999, 32), BASE_SEED + 4, silu_qk=True)
    if name == "c5":
        lam = [1.0] * 16 + lambda_geometric(0.95, 0.9999, 16)
        return Workload("c5", "bf16", 1, 32, 131072, 128, lam, BASE_SEED + 5)
    raise KeyError(name)


def c3_sweep() -> List[Workload]:
    return [workload("c3_%d" % n) for (_, n) in _c3_points()]


def custom(B: int, H: int, n: int, d: int, lambdas: Sequence[float], seed: int,
           dtype: str = "f32", silu_qk: bool = False, name: str = "custom") -> Workload:
    assert len(lambdas) == H
    return Workload(name, dtype, B, H, n, d, [float(x) for x in lambdas], seed, silu_qk)


def draw(w: Workload, heads: Optional[Sequence[int]] = None,
         batches: Optional[Sequence[int]] = None):
    """Draw (Q, K, V, dO) as fp32 CPU tensors for workload `w`.

    The full tensors are always drawn (so that a sub-selection sees the same
    values as the full workload); `heads` / `batches` then select slices.
    For large workloads prefer `draw_on(...)`, which generates per (b, h) slab.
    """
    g = torch.Generator(device="cpu").manual_seed(w.seed)
    shape = (w.B, w.H, w.n, w.d)
    s = 1.0 / math.sqrt(w.d)
    out = []
    for i in range(4):
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        if i < 3:
            if w.silu_qk and i < 2:
                x = torch.nn.functional.silu(x)
            x = x * s
        out.append(x)
    if batches is not None:
        out = [x[list(batches)] for x in out]
    if heads is not None:
        out = [x[:, list(heads)] for x in out]
    return tuple(x.contiguous() for x in out)


def slab_seed(w: Workload, tensor_index: int, b: int, h: int) -> int:
    """Seed of one (tensor, b, h) slab for the slab-wise generator."""
    return (w.seed * 1000003 + tensor_index * 7919 + b * 104729 + h * 1299709) % (2 ** 31 - 1)


def draw_slab(w: Workload, tensor_index: int, b: int, h: int) -> torch.Tensor:
    """One `[n, d]` fp32 slab of tensor `tensor_index` (0=Q, 1=K, 2=V, 3=dO).

    Slab-wise generation lets a test rebuild any single (b, h) scan of a large
    workload on the host without materialising the whole tensor.
    """
    g = torch.Generator(device="cpu").manual_seed(slab_seed(w, tensor_index, b, h))
    x = torch.randn((w.n, w.d), generator=g, dtype=torch.float32)
    if tensor_index < 3:
        if w.silu_qk and tensor_index < 2:
            x = torch.nn.functional.silu(x)
        x = x * (1.0 / math.sqrt(w.d))
    return x


def draw_slabwise(w: Workload, device: str = "cpu", dtype: torch.dtype = torch.float32):
    """Draw (Q, K, V, dO) slab by slab (values differ from `draw`, same
    distribution), placing each slab directly into a tensor on `device`."""
    out = []
    for ti in range(4):
        t = torch.empty((w.B, w.H, w.n, w.d), dtype=dtype, device=device)
        for b in range(w.B):
            for h in range(w.H):
                t[b, h].copy_(draw_slab(w, ti, b, h).to(dtype))
        out.append(t)
    return tuple(out)
