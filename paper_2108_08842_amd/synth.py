"""Seeded synthetic inputs with the shapes and value distributions of the paper's workloads.

Holds none of the method's arithmetic: only input vectors, bit budgets and drop rates.  Both the HIP
path (tests, benchmark) and the CPU oracle's checks draw their inputs from here.

Workloads (they stand in for the paper's own experiments, whose datasets and trained models are not
used here): i.i.d. normal vectors; LogNormal(0,1) vectors as in the paper's vNMSE / encoding-speed
experiment (Sec. 5.2); a vector of the size of a ResNet-18 gradient made of 64 "layers" with very
different scales (App. F, NMSE experiment shape); normal vectors with rare large outliers; per-client
mixed budgets with 10% packet loss (Sec. 4.1, 4.2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


@dataclass
class Workload:
    name: str
    n: int                      # senders
    d: int                      # coordinates per sender
    b_q8: List[int]             # per-sender bit budget, 256 = one bit per coordinate
    seed: int                   # the round's shared seed
    dist: str                   # value distribution, see client_vector
    drop_q32: int = 0           # per-packet drop probability * 2^32 (0 = lossless)
    client_ids: List[int] = field(default_factory=list)

    def __post_init__(self):
        if not self.client_ids:
            self.client_ids = list(range(self.n))


def _rng(workload_seed: int, client: int) -> np.random.Generator:
    return np.random.default_rng([0xEDE0, workload_seed & 0xFFFFFFFF, client])


def client_vector(w: Workload, c: int, d: Optional[int] = None) -> np.ndarray:
    """fp32 vector of sender c.  `d` overrides the workload's dimension (scaled-down parity cases)."""
    d = w.d if d is None else d
    rng = _rng(w.seed, w.client_ids[c])
    if w.dist == "normal":
        x = rng.standard_normal(d, dtype=np.float32)
    elif w.dist == "lognormal_signed":
        x = np.exp(rng.standard_normal(d, dtype=np.float32))
        x *= rng.integers(0, 2, d, dtype=np.int8).astype(np.float32) * 2.0 - 1.0
    elif w.dist == "lognormal":
        x = np.exp(rng.standard_normal(d, dtype=np.float32))
    elif w.dist == "layers":
        # 64 contiguous blocks of random sizes, block l ~ N(0, sigma_l^2), sigma_l log-uniform in [1e-4, 1e-1]
        cuts = np.sort(rng.integers(1, d, 63)) if d > 64 else np.arange(1, min(d, 64))
        edges = np.concatenate([[0], cuts, [d]])
        sigma = np.exp(rng.uniform(np.log(1e-4), np.log(1e-1), edges.size - 1)).astype(np.float32)
        x = rng.standard_normal(d, dtype=np.float32)
        for l in range(edges.size - 1):
            x[edges[l]:edges[l + 1]] *= sigma[l]
    elif w.dist == "normal_outliers":
        x = rng.standard_normal(d, dtype=np.float32)
        k = max(1, d // 1000)
        x[rng.integers(0, d, k)] *= 100.0
    else:
        raise ValueError(w.dist)
    return np.ascontiguousarray(x, dtype=np.float32)


def _mixed_budgets(n: int, seed: int) -> List[int]:
    rng = np.random.default_rng([0xB0D6, seed])
    return [int(v) for v in rng.choice([128, 256, 512, 1024], n)]


def config(i: int) -> Workload:
    """The five synthetic configurations the throughput metric is defined on (1-based)."""
    if i == 1:
        return Workload("cfg1_n4_d1024_b1", 4, 1024, [256] * 4, 0, "normal")
    if i == 2:
        return Workload("cfg2_n10_d2^20_b2", 10, 1 << 20, [512] * 10, 2, "lognormal_signed")
    if i == 3:
        return Workload("cfg3_n32_d2^20_mixed_loss10", 32, 1 << 20, _mixed_budgets(32, 3), 3, "lognormal",
                        drop_q32=int(0.1 * 2 ** 32))
    if i == 4:
        return Workload("cfg4_n16_d11173962_b1", 16, 11_173_962, [256] * 16, 4, "layers")
    if i == 5:
        return Workload("cfg5_n8_d2^27_b4", 8, 1 << 27, [1024] * 8, 5, "normal_outliers")
    raise ValueError("config index must be 1..5")
