"""Synthetic workloads: matrix shapes and seeded input generators.

Holds none of the method's arithmetic (no projection, no generator for A, no
compress/decompress): only the shapes of the five benchmark configurations and
seeded torch recipes for gradients and weights.  Tests hand the same tensors
to the GPU library and to the CPU oracle.

The paper trains T5 and GPT-2 models on public corpora (Section 3.1); those
datasets and checkpoints are not used here.  These inputs stand in for them
and borrow only the models' weight-matrix shapes (hidden sizes 512, 1024,
768, 1600 as stated in Section 3.1, "Models").
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Tuple

import torch


@dataclass
class Workload:
    index: int
    name: str
    shapes: List[Tuple[int, int]]          # (n, m) per matrix; m is the compressed axis
    grad_dtype: str                        # "f32" | "bf16"
    r: int
    algorithm: int                         # 1 = accumulation (Alg. 1), 2 = momentum (Alg. 2)
    tau: int = 1                           # Alg. 1: micro-steps per cycle
    beta: float = 0.0                      # Alg. 2
    kappa: int = 0                         # Alg. 2: resampling interval
    steps: int = 1                         # Alg. 2: steps in the schedule
    lr: float = 1e-3
    rule: str = "sgd"                      # "sgd" | "factored"
    grad_kind: str = "normal"
    grad_rank: int = 0
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def elements(self) -> int:
        return sum(n * m for n, m in self.shapes)

    @property
    def grad_bytes(self) -> int:
        return self.elements * (4 if self.grad_dtype == "f32" else 2)

    @property
    def state_elements(self) -> int:
        return sum(n * self.r for n, _ in self.shapes)


def _t5_small_shapes():
    d, ff = 512, 2048
    s = []
    for _ in range(6):                      # encoder: q k v o
        s += [(d, d)] * 4 + [(ff, d), (d, ff)]
    for _ in range(6):                      # decoder: self q k v o + cross q k v o
        s += [(d, d)] * 8 + [(ff, d), (d, ff)]
    return s


def _gpt2_shapes(layers, d):
    s = []
    for _ in range(layers):
        s += [(d, 3 * d), (d, d), (d, 4 * d), (4 * d, d)]
    return s


def _t5_3b_shapes():
    d, inner, ff = 1024, 4096, 16384
    s = []
    for _ in range(24):                     # encoder: q k v (d x inner), o (inner x d)
        s += [(d, inner)] * 3 + [(inner, d), (d, ff), (ff, d)]
    for _ in range(24):                     # decoder: self + cross attention
        s += [(d, inner)] * 6 + [(inner, d)] * 2 + [(d, ff), (ff, d)]
    return s


def workload(index: int) -> Workload:
    if index == 1:
        return Workload(1, "single-256x256-f32-r8", [(256, 256)], "f32", 8, 1, tau=4,
                        grad_kind="normal", seed=0)
    if index == 2:
        return Workload(2, "t5-small-f32-r16-tau8", _t5_small_shapes(), "f32", 16, 1, tau=8,
                        grad_kind="lowrank+noise", grad_rank=16, seed=2)
    if index == 3:
        return Workload(3, "gpt2-base-bf16-r64-momentum", _gpt2_shapes(12, 768), "bf16", 64, 2,
                        beta=0.9, kappa=100, steps=300, grad_kind="row-lognormal", seed=3)
    if index == 4:
        return Workload(4, "t5-3b-bf16-r256-tau16-factored", _t5_3b_shapes(), "bf16", 256, 1,
                        tau=16, rule="factored", grad_kind="lowrank+noise", grad_rank=32, seed=4,
                        extra=dict(beta2=0.0, eps1=1e-30, clip_d=1.0))
    if index == 5:
        return Workload(5, "gpt2-xl-bf16-r256-momentum-fused", _gpt2_shapes(48, 1600), "bf16", 256,
                        2, beta=0.9, kappa=1000, steps=2000, grad_kind="student-t3", seed=5)
    raise ValueError("workload index must be 1..5")


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_generator(seed: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_grad(wl: Workload, n: int, m: int, gen: torch.Generator, device="cpu") -> torch.Tensor:
    """One gradient matrix of the workload's distribution, in its dtype."""
    kind = wl.grad_kind
    f32 = torch.float32
    if kind == "normal":
        g = torch.randn(n, m, generator=gen, device=device, dtype=f32)
    elif kind == "lowrank+noise":
        k = wl.grad_rank
        u = torch.randn(n, k, generator=gen, device=device, dtype=f32)
        v = torch.randn(m, k, generator=gen, device=device, dtype=f32)
        g = (u @ v.t()) / math.sqrt(k)
        g += 0.1 * torch.randn(n, m, generator=gen, device=device, dtype=f32)
    elif kind == "row-lognormal":
        z = torch.randn(n, 1, generator=gen, device=device, dtype=f32)
        g = torch.exp(z) * torch.randn(n, m, generator=gen, device=device, dtype=f32)
    elif kind == "student-t3":
        num = torch.randn(n, m, generator=gen, device=device, dtype=f32)
        den = torch.zeros(n, m, device=device, dtype=f32)
        for _ in range(3):
            den += torch.randn(n, m, generator=gen, device=device, dtype=f32) ** 2
        g = num / torch.sqrt(den / 3.0)
    else:
        raise ValueError(kind)
    return g.to(torch_dtype(wl.grad_dtype)).contiguous()


def make_weight(n: int, m: int, gen: torch.Generator, device="cpu") -> torch.Tensor:
    return torch.randn(n, m, generator=gen, device=device, dtype=torch.float32).contiguous()


def make_grad_set(wl: Workload, gen: torch.Generator, device="cpu") -> List[torch.Tensor]:
    return [make_grad(wl, n, m, gen, device) for (n, m) in wl.shapes]


def make_weight_set(wl: Workload, gen: torch.Generator, device="cpu") -> List[torch.Tensor]:
    return [make_weight(n, m, gen, device) for (n, m) in wl.shapes]
