"""Seeded synthetic sparse tensors with the shapes of the paper's workloads.

This module is the only thing the CPU oracle's tests and the HIP path's tests
share.  It holds no arithmetic of the method: it only draws COO coordinates and
values (numpy, Philox bit generator, fully determined by the seed) and names the
five benchmark workloads.  The real rating datasets the paper measures on
(Section 5.1, Table of real world datasets) are not available; the workloads
below imitate their shapes, sizes and value ranges with synthetic draws.

Coordinates of a skewed mode follow a bounded, discretised power law
  rank = floor((1 + u * ((I + 1)^(1 - s) - 1))^(1 / (1 - s))) - 1,  u ~ U[0, 1)
and ranks are scattered over row ids by the bijection  i = (a * rank + b) mod I
with gcd(a, I) = 1, so that frequently hit rows are not neighbours in memory.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dims: Tuple[int, ...]
    nnz: int
    J: Tuple[int, ...]
    R: int
    n_samples: int                      # |Psi| per step
    zipf: Tuple[Optional[float], ...]   # per mode: exponent s, or None for uniform
    values: str                         # "int1to5" | "int0to100_scaled" | "normal"
    distinct: bool = False              # coordinates drawn without repetition
    lr_A: float = 1e-3
    lr_B: float = 1e-3
    lambda_A: float = 1e-2
    lambda_B: float = 1e-2
    data_seed: int = 0
    init_seed: int = 1
    sample_seed0: int = 1000            # step t uses seed sample_seed0 + t

    @property
    def order(self) -> int:
        return len(self.dims)

    def scaled(self, nnz: int, n_samples: int, dims: Optional[Tuple[int, ...]] = None) -> "Workload":
        """Same recipe at a smaller size (for tests the oracle finishes in seconds)."""
        return replace(self, nnz=int(nnz), n_samples=int(n_samples),
                       dims=tuple(dims) if dims is not None else self.dims,
                       name=self.name + "-scaled")


# Step sizes: C1's are given (1e-3).  With U(0, 0.5) parameters the starting
# prediction is about R (J/16)^N and a frequently hit row collects ~1e5 gradients
# per step (M = 1 for factor rows), so the larger workloads need far smaller
# steps to stay finite; throughput does not depend on them.
WORKLOADS = {
    "C1": Workload("C1", (1000, 800, 600), 100_000, (8, 8, 8), 8, 10_000,
                   (None, None, None), "int1to5", distinct=True,
                   lr_A=1e-3, lr_B=1e-3, data_seed=101),
    "C2": Workload("C2", (480_000, 17_770, 2_200), 100_000_000, (16, 16, 16), 16, 1_000_000,
                   (1.1, 1.1, None), "int1to5", lr_A=2e-10, lr_B=1e-4, data_seed=102),
    "C3": Workload("C3", (1_000_000, 625_000, 3_000), 250_000_000, (32, 32, 32), 32, 4_000_000,
                   (1.2, 1.2, None), "int0to100_scaled", lr_A=1e-13, lr_B=1e-10, data_seed=103),
    "C4": Workload("C4", (100_000,) * 6, 200_000_000, (8,) * 6, 16, 2_000_000,
                   (None,) * 6, "normal", lr_A=1e-3, lr_B=1e-3, data_seed=104),
    "C5": Workload("C5", (480_000, 17_770, 2_200), 100_000_000, (64, 64, 64), 64, 1_000_000,
                   (1.1, 1.1, None), "int1to5", lr_A=1e-15, lr_B=1e-12, data_seed=105),
}


# The paper's order-scalability sweep (Section 5.4, synthetic data table): orders 5..10, 10 000 rows per mode,
# 1e8 stored entries with values 1..5; it reports the sweep for J_n = R = 4.  With U(0, 0.5) parameters and
# J = R = 4 the starting prediction is 4 / 4^N: tiny, so plain step sizes are stable.
for _n in range(5, 11):
    WORKLOADS["O%d" % _n] = Workload("O%d" % _n, (10_000,) * _n, 100_000_000, (4,) * _n, 4, 1_000_000,
                                     (None,) * _n, "int1to5", lr_A=1e-3, lr_B=1e-3, data_seed=200 + _n)


def _coprime_multiplier(I: int) -> int:
    a = max(1, int(round(0.6180339887 * I)))
    while math.gcd(a, I) != 1:
        a += 1
    return a


def scatter_params(I: int) -> Tuple[int, int]:
    """(a, b) of the rank -> row-id bijection i = (a * rank + b) mod I."""
    return _coprime_multiplier(I), I // 3


def _zipf_mode(rng: np.random.Generator, count: int, I: int, s: float) -> np.ndarray:
    out = np.empty(count, dtype=np.int32)
    a, b = scatter_params(I)
    span = (I + 1.0) ** (1.0 - s) - 1.0
    inv = 1.0 / (1.0 - s)
    chunk = 1 << 24
    for lo in range(0, count, chunk):
        hi = min(count, lo + chunk)
        u = rng.random(hi - lo)
        rank = np.floor((1.0 + u * span) ** inv).astype(np.int64) - 1
        np.clip(rank, 0, I - 1, out=rank)
        out[lo:hi] = ((a * rank + b) % I).astype(np.int32)
    return out


def _values(rng: np.random.Generator, count: int, kind: str) -> np.ndarray:
    if kind == "int1to5":
        return rng.integers(1, 6, size=count, dtype=np.int32).astype(np.float32)
    if kind == "int0to100_scaled":
        return rng.integers(0, 101, size=count, dtype=np.int32).astype(np.float32) / np.float32(100.0)
    if kind == "normal":
        return rng.standard_normal(size=count, dtype=np.float32)
    raise ValueError("unknown value kind %r" % kind)


def make_tensor(w: Workload) -> Tuple[List[np.ndarray], np.ndarray]:
    """COO of the workload: (idx[n] int32[nnz] for each mode, vals float32[nnz])."""
    N = w.order
    idx: List[np.ndarray] = []
    if w.distinct:
        total = 1
        for d in w.dims:
            total *= int(d)
        if w.nnz > total:
            raise ValueError("more distinct coordinates asked for than cells exist")
        rng = np.random.Generator(np.random.Philox(key=w.data_seed))
        lin = np.empty(0, dtype=np.int64)
        while lin.shape[0] < w.nnz:
            extra = rng.integers(0, total, size=int(1.2 * (w.nnz - lin.shape[0])) + 16, dtype=np.int64)
            lin = np.unique(np.concatenate([lin, extra]))
        lin = rng.permutation(lin)[: w.nnz]
        rem = lin
        cols = []
        for n in range(N - 1, -1, -1):
            cols.append((rem % w.dims[n]).astype(np.int32))
            rem = rem // w.dims[n]
        idx = [np.ascontiguousarray(c) for c in cols[::-1]]
    else:
        for n in range(N):
            rng = np.random.Generator(np.random.Philox(key=[w.data_seed, n]))
            if w.zipf[n] is None:
                idx.append(rng.integers(0, w.dims[n], size=w.nnz, dtype=np.int32))
            else:
                idx.append(_zipf_mode(rng, w.nnz, int(w.dims[n]), float(w.zipf[n])))
    rng_v = np.random.Generator(np.random.Philox(key=[w.data_seed, 15]))
    vals = _values(rng_v, w.nnz, w.values)
    return idx, vals


def tiny_workload(order: int, dims, nnz: int, J, R: int, n_samples: int, seed: int = 7,
                  values: str = "normal", zipf=None) -> Workload:
    """Hand-sized workload for unit tests (arbitrary, also non-uniform, ranks)."""
    return Workload("tiny", tuple(int(d) for d in dims), int(nnz), tuple(int(j) for j in J), int(R),
                    int(n_samples), tuple(zipf) if zipf is not None else (None,) * order, values,
                    data_seed=seed, init_seed=seed + 1)
