"""The synthetic workloads: shapes, worker counts and hyper-parameters.

Hyper-parameters follow the paper's experiments (Section 4, Appendix A.2-A.4:
Nesterov momentum 0.9, weight decay 1e-4, tau = 12 for Local SGD, alpha = 1,
beta in 0.4..0.8; Adam with beta1 0.9, beta2 0.98, eps 1e-8).  Gradients and
initial parameters are seeded synthetic values (generator.py) standing in for
CIFAR-10 / ImageNet / WMT'16 training, which need data that is not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from . import shapes as _shapes

BASE_SEED = 191000643


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                     # position in the benchmark's config list
    shapes: tuple
    m: int
    tau: int
    alpha: float
    beta: float
    base: str                      # "sgd_nesterov" | "adam"
    policy: str                    # "reset" | "maintain"
    lr: float
    momentum: float = 0.0
    weight_decay: float = 0.0
    beta1: float = 0.9
    beta2: float = 0.98
    eps: float = 1e-8
    grad_dtype: str = "f32"        # "f32" | "bf16"
    sigma: float = 1.0             # gradient standard deviation
    rounds: int = 3
    exact_average: bool = True     # False: the variant without line 6 of Algorithm 1 (Section 6)
    mix: str = "none"              # a gossip step (Appendix C.1) after every local step:
                                   # "expgraph" (one-peer exponential graph) or "random"
                                   # (in_peers below: any map, so push-sum weights move)
    tensor_wd: tuple | None = None        # per-tensor weight decay (else weight_decay for all)
    tensor_lr_scale: tuple | None = None  # per-tensor factor on the fast learning rate

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def numel(self) -> List[int]:
        return _shapes.numels(list(self.shapes))

    @property
    def d(self) -> int:
        return sum(self.numel)

    @property
    def tensor_starts(self) -> np.ndarray:
        """Global element index of the first element of every tensor (the
        tensors are numbered consecutively, without padding)."""
        n = np.asarray(self.numel, dtype=np.int64)
        return np.concatenate([[0], np.cumsum(n)[:-1]]).astype(np.int64)

    @property
    def updates_per_round(self) -> int:
        return self.m * self.d * self.tau

    def f32(self, name: str) -> float:
        """A hyper-parameter as the fp32 value that crosses the C boundary,
        widened to a Python float; both sides compute with exactly this."""
        return float(np.float32(getattr(self, name)))


def tiny() -> Workload:
    return Workload("tiny", 0, tuple(_shapes.tiny_flat()), m=4, tau=12, alpha=1.0,
                    beta=0.7, base="sgd_nesterov", policy="reset", lr=0.1,
                    momentum=0.9, weight_decay=1e-4, sigma=1.0, rounds=10)


def resnet18() -> Workload:
    return Workload("resnet18", 1, tuple(_shapes.resnet18()), m=8, tau=12, alpha=1.0,
                    beta=0.6, base="sgd_nesterov", policy="reset", lr=0.1,
                    momentum=0.9, weight_decay=1e-4, sigma=0.1, rounds=20)


def resnet50() -> Workload:
    return Workload("resnet50", 2, tuple(_shapes.resnet50()), m=32, tau=12, alpha=1.0,
                    beta=0.6, base="sgd_nesterov", policy="reset", lr=0.1,
                    momentum=0.9, weight_decay=1e-4, sigma=0.1, rounds=20)


def transformer_big() -> Workload:
    return Workload("transformer_big", 3, tuple(_shapes.transformer_big()), m=8, tau=48,
                    alpha=1.0, beta=0.5, base="adam", policy="maintain", lr=5e-4,
                    beta1=0.9, beta2=0.98, eps=1e-8, grad_dtype="bf16", sigma=0.1,
                    rounds=3)


def stress() -> Workload:
    return Workload("stress", 4, tuple(_shapes.stress_flat()), m=8, tau=48, alpha=1.0,
                    beta=0.7, base="sgd_nesterov", policy="reset", lr=0.05,
                    momentum=0.9, weight_decay=0.0, sigma=1.0, rounds=3)


def ragged_mini(base: str = "sgd_nesterov", grad_dtype: str = "f32", m: int = 3,
                policy: str | None = None) -> Workload:
    """Small multi-tensor case for element-by-element parity (not a benchmark)."""
    if base == "adam":
        return Workload("ragged_mini_adam", 7, tuple(_shapes.ragged_mini()), m=m, tau=5,
                        alpha=1.0, beta=0.5, base="adam", policy=policy or "maintain",
                        lr=5e-4, grad_dtype=grad_dtype, sigma=0.1, rounds=4)
    return Workload("ragged_mini_sgd", 6, tuple(_shapes.ragged_mini()), m=m, tau=5,
                    alpha=0.75, beta=0.6, base="sgd_nesterov", policy=policy or "reset",
                    lr=0.1, momentum=0.9, weight_decay=1e-4, grad_dtype=grad_dtype,
                    sigma=0.1, rounds=4)


def in_peers(w: Workload, step: int) -> np.ndarray:
    """Seeded in-neighbour map for mix == "random": worker i receives from
    in_peers[i] (itself: from nobody).  Any map may come out: several receivers
    per sender, chains, cycles, idle workers."""
    rng = np.random.default_rng([w.seed, 0x6d6978, step])
    return rng.integers(0, w.m, size=w.m).astype(np.int32)


BY_NAME = {"tiny": tiny, "resnet18": resnet18, "resnet50": resnet50,
           "transformer_big": transformer_big, "stress": stress}
