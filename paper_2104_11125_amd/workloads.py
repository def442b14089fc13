"""Seeded synthetic workloads: shapes and gradient generators only.

This module holds none of the method's arithmetic.  It is the one piece shared by the GPU
tests, the benchmark and the oracle-side tests: it produces the bytes that both the HIP
library and the CPU oracle consume.

The gradients stand in for the per-learner gradients of the paper's workloads (ResNet50 /
ImageNet at 112X, Transformer-base / WMT14 and the speech LSTM at 400X, Sec. 4 and Tables 2
and 3), which cannot be produced here.  What is kept from them: the vector lengths, the
number of learners, the compression rates, and the premise of Sec. 2 that learners'
gradients are similar, modelled as a component shared by all learners plus independent
per-learner noise:  g_i = 1e-3 * (s + c * e_i).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int            # enters the seeds
    n_learners: int
    numel: int             # length of each learner's flat vector
    rate: int              # compression rate: k = numel // rate (flat) or ceil(size / rate) per tensor
    noise: float           # c in g_i = 1e-3 * (s + c * e_i)
    dist: str              # "normal" or "student_t3"
    beta: float
    lr: float
    steps: int
    grad_dtype: str = "f32"             # "f32" or "bf16"
    n_tensors: int = 1                  # > 1: per-tensor index sets
    offsets: Optional[tuple] = field(default=None)   # n_tensors + 1 segment boundaries
    ks: Optional[tuple] = field(default=None)        # per-tensor k

    @property
    def k(self) -> int:
        return self.numel // self.rate if self.n_tensors == 1 else int(sum(self.ks))


def _layer_sizes(seed: int, n_tensors: int, lo: int, hi: int) -> List[int]:
    """Sizes log-uniform on [lo, hi]: round(lo * (hi / lo) ** u), u ~ U[0, 1)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    u = torch.rand(n_tensors, generator=g, dtype=torch.float64)
    return [int(round(lo * (hi / lo) ** float(x))) for x in u]


def per_layer_workload(name="per_layer", cfg_id=4, n_learners=8, n_tensors=200, lo=64, hi=4_194_304, rate=100,
                       steps=5, seed=4004) -> Workload:
    sizes = _layer_sizes(seed, n_tensors, lo, hi)
    offsets = [0]
    for s in sizes:
        offsets.append(offsets[-1] + s)
    ks = [int(math.ceil(s / rate)) for s in sizes]
    return Workload(name, cfg_id, n_learners, offsets[-1], rate, 0.5, "normal", 0.1, 0.1, steps, "f32",
                    n_tensors, tuple(offsets), tuple(ks))


def configs() -> List[Workload]:
    """The five benchmark configurations, in the order they are numbered."""
    return [
        Workload("tiny", 1, 4, 1_048_576, 100, 0.3, "normal", 0.1, 0.1, 3),
        Workload("resnet50_sized", 2, 8, 25_557_032, 112, 0.5, "normal", 0.1, 0.1, 10),
        Workload("transformer_base_sized", 3, 16, 110_000_000, 400, 0.5, "student_t3", 0.2, 0.05, 10),
        per_layer_workload(),
        Workload("large_bf16", 5, 8, 1_000_000_000, 400, 0.5, "normal", 0.1, 0.1, 3, "bf16"),
    ]


def by_name(name: str) -> Workload:
    for w in configs():
        if w.name == name:
            return w
    raise KeyError(name)


def scaled(w: Workload, numel: int, n_learners: Optional[int] = None, steps: Optional[int] = None) -> Workload:
    """Same recipe at another length (flat workloads only): used for parity cases small
    enough for the oracle."""
    assert w.n_tensors == 1
    return Workload(f"{w.name}@{numel}", w.cfg_id, n_learners or w.n_learners, numel, w.rate, w.noise, w.dist,
                    w.beta, w.lr, steps or w.steps, w.grad_dtype)


def _seed(cfg_id: int, step: int, learner: int) -> int:
    # learner = -1 is the shared component
    return (cfg_id * 1000 + step) * 1000 + (learner + 1)


def _draw(dist: str, numel: int, gen: torch.Generator, device) -> torch.Tensor:
    if dist == "normal":
        return torch.randn(numel, generator=gen, device=device, dtype=torch.float32)
    if dist == "student_t3":
        # t with 3 degrees of freedom: z0 / sqrt((z1^2 + z2^2 + z3^2) / 3)
        z0 = torch.randn(numel, generator=gen, device=device, dtype=torch.float32)
        den = torch.zeros(numel, device=device, dtype=torch.float32)
        for _ in range(3):
            z = torch.randn(numel, generator=gen, device=device, dtype=torch.float32)
            den.addcmul_(z, z)
        den.div_(3.0).sqrt_()
        return z0.div_(den)
    raise ValueError(dist)


def shared_component(w: Workload, step: int, device) -> torch.Tensor:
    gen = torch.Generator(device=device)
    gen.manual_seed(_seed(w.cfg_id, step, -1))
    return _draw(w.dist, w.numel, gen, device)


def learner_gradient(w: Workload, step: int, learner: int, device, shared: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """g_i = 1e-3 * (s + c * e_i) in float32, then rounded to bfloat16 (round to nearest
    even) when the workload stores gradients in bfloat16."""
    s = shared if shared is not None else shared_component(w, step, device)
    gen = torch.Generator(device=device)
    gen.manual_seed(_seed(w.cfg_id, step, learner))
    e = _draw(w.dist, w.numel, gen, device)
    e.mul_(w.noise).add_(s).mul_(1e-3)
    g = e.to(torch.bfloat16) if w.grad_dtype == "bf16" else e
    if out is not None:
        out.copy_(g)
        return out
    return g


def gradients(w: Workload, step: int, device, out: Optional[List[torch.Tensor]] = None) -> List[torch.Tensor]:
    """All learners' gradients of one step (fresh draws every step)."""
    s = shared_component(w, step, device)
    res = []
    for i in range(w.n_learners):
        res.append(learner_gradient(w, step, i, device, shared=s, out=None if out is None else out[i]))
    return res


def zero_memories(w: Workload, device) -> List[torch.Tensor]:
    """Memories start at zero (Alg. 1, input line)."""
    return [torch.zeros(w.numel, device=device, dtype=torch.float32) for _ in range(w.n_learners)]
