"""Seeded random instances of the resource-allocation problem (Sec. III-B).

An instance is plain data: total CU count T, the sorted configuration list, and per
worker the kernels-per-unit counts and the integer latency table beta[unit][config]
in nanoseconds.  No objective arithmetic lives here."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

OVERLAP_EXCESS, OVERLAP_LITERAL, OVERLAP_TABLE = range(3)


@dataclass
class Worker:
    n_kernels: List[int]                 # kernels per unit, in execution order
    beta: List[List[int]]                # beta[unit][config index], integer ns


@dataclass
class AllocProblem:
    total_cus: int
    configs: List[int]                   # strictly increasing CU counts
    workers: List[Worker]
    switch_max: int
    overlap_mode: int = OVERLAP_EXCESS
    alpha_ppm: Optional[List[int]] = None   # TABLE mode: non-decreasing slowdown (ppm) per overlap granule
    granule: int = 1                        # TABLE mode: CUs per granule
    max_configs: int = 0                    # distinct configurations a worker may use (0 = no limit)
    switch_cost: int = 0                    # ns added to a worker's time per configuration switch
    max_configs_w: Optional[List[int]] = None   # per-worker limits on distinct configurations (replace max_configs)


def random_problem(seed: int, n_workers: int, units: List[int], configs: List[int], total_cus: int,
                   switch_max: int, mode: int = OVERLAP_EXCESS, shape: str = "scaling",
                   max_kernels: int = 4) -> AllocProblem:
    """`shape`: 'scaling' = latency falls with CU count down to a random knee (the usual profile),
    'random' = unrelated integers, 'flat' = independent of the CU count, 'ties' = tiny value range."""
    rng = np.random.default_rng(seed)
    workers = []
    for w in range(n_workers):
        g = units[w]
        n_k = [int(rng.integers(1, max_kernels + 1)) for _ in range(g)]
        beta = []
        for u in range(g):
            if shape == "flat":
                v = int(rng.integers(1000, 100000))
                row = [v] * len(configs)
            elif shape == "random":
                row = [int(rng.integers(1, 100000)) for _ in configs]
            elif shape == "ties":
                row = [int(rng.integers(1, 4)) for _ in configs]
            else:
                work = float(rng.integers(2000, 400000))
                knee = configs[int(rng.integers(0, len(configs)))]
                floor = float(rng.integers(500, 5000))
                row = [int(floor + work * knee / min(c, knee) / 8.0) for c in configs]
            beta.append(row)
        workers.append(Worker(n_k, beta))
    alpha = None
    granule = 1
    if mode == OVERLAP_TABLE:
        granule = configs[0]
        n = (n_workers * total_cus) // granule + 2
        steps = rng.integers(0, 200000, size=n)
        alpha = [int(v) for v in np.cumsum(steps)]
        alpha[0] = 0
    return AllocProblem(total_cus, list(configs), workers, switch_max, mode, alpha, granule)
