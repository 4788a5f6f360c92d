"""Allocation oracle: exhaustive search over the paper's resource-allocation model.

TEST INFRASTRUCTURE ONLY (tests, smoke check, CPU-baseline timing).  Shares no code
with the library's solver.

Model (Sec. III-B, "Optimization Formulation"), lifted from kernels to *units*: a
unit is a run of n >= 1 consecutive kernels that must share one CU configuration
(n = 1 everywhere gives the paper's per-kernel model).

  * every unit takes exactly one configuration (one-hot x, first constraint);
  * switchTotal_w counts the positions where consecutive units differ (second
    constraint; the printed |x - x'|/2 sum is the same number) and must not exceed
    switchMax (third constraint); the first unit has no predecessor and is free;
  * beta = profiled solo latency of the unit at its configuration;
  * CUAverage_w = (sum over kernels of the CU count they run on) / (#kernels of w);
  * alpha = CUOverlap / total CUs, the same for every worker, and e = beta*(1+alpha);
  * objective = unweighted sum over workers of sum of e.

Readings where the text is ambiguous (each is a mode or rule below, never silent):
  EXCESS   CUOverlap = max(0, sum_w CUAverage_w - T): the overlap a disjoint-first
           mask layout produces (the two-worker mask example of Sec. III-A overlaps in
           exactly that many CUs for all nine size pairs) and the only reading under
           which "two identical kernels sharing the same CUs take twice as long" gives
           alpha = 1 while a lone worker gets alpha = 0.
  LITERAL  CUOverlap = sum_w CUAverage_w, the formula exactly as printed.
  TABLE    alpha comes from a measured non-decreasing table (parts per million) indexed
           by floor(EXCESS overlap / granule).
  Ties: smaller sum of CU averages first (fewer CUs), then the lexicographically
  smallest vector of configuration indices, worker-major, unit order.

Two extensions beyond the printed model, both off (0) by default so that the paper's model is the
special case:
  max_configs  a worker may use at most this many *distinct* configurations in one request (max_configs_w: the same
               limit given per worker, so that a global stream budget can be split unevenly).  It is the
               stream-pool limit of Sec. III-A turned into a constraint: every (worker, configuration)
               pair in use is one pooled stream, and the GPU runs only a few streams without
               oversubscribing its hardware queues (7 on the paper's MI50; 4 on MI355X, one per pipe).
  switch_cost  nanoseconds added to a worker's solo time per configuration switch: factor (iii) of
               Sec. III-B (what a change of CU configuration costs), which the paper bounds with the
               budget only; with a cost the optimizer stops switching for gains smaller than a switch.

All arithmetic is exact (Python integers).  With D = lcm_w(N_w), S_D = D * sum_w
CUAverage_w is an integer, and the objective is compared through the integer
  EXCESS/LITERAL:  (sum_w B_w) * (T*D + Ov_D)        (= objective * T * D)
  TABLE:           (sum_w B_w) * (10**6 + alpha_ppm)  (= objective * 10**6)
"""
from __future__ import annotations

import itertools
from math import gcd
from typing import List, Optional, Sequence, Tuple

OVERLAP_EXCESS, OVERLAP_LITERAL, OVERLAP_TABLE = range(3)


def _lcm(a, b):
    return a // gcd(a, b) * b


def switch_total(cfg_idx: Sequence[int]) -> int:
    """Number of configuration switches of one worker: positions g >= 1 whose configuration
    differs from the previous unit's."""
    return sum(1 for g in range(1, len(cfg_idx)) if cfg_idx[g] != cfg_idx[g - 1])


def switch_total_onehot(cfg_idx: Sequence[int], n_configs: int) -> int:
    """The same count through the printed one-hot form: sum_k sum_c |x[k][c] - x[k-1][c]| / 2."""
    x = [[1 if c == ci else 0 for c in range(n_configs)] for ci in cfg_idx]
    tot = 0
    for k in range(1, len(x)):
        tot += sum(abs(x[k][c] - x[k - 1][c]) for c in range(n_configs))
    assert tot % 2 == 0
    return tot // 2


def evaluate(p, assign: Sequence[Sequence[int]]):
    """Exact evaluation of one assignment (list per worker of configuration indices).

    Returns None when a worker exceeds the switch budget, else
    (objective_numerator, S_D, switches_per_worker)."""
    switches = [switch_total(a) for a in assign]
    if any(s > p.switch_max for s in switches):
        return None
    max_configs = getattr(p, "max_configs", 0)
    per_worker = getattr(p, "max_configs_w", None)          # per-worker limits replace the common one (0 = no limit)
    limits = list(per_worker) if per_worker is not None else [max_configs] * len(assign)
    if any(lim and len(set(a)) > lim for a, lim in zip(assign, limits)):
        return None
    switch_cost = getattr(p, "switch_cost", 0)
    T = p.total_cus
    n_tot = [sum(w.n_kernels) for w in p.workers]
    D = 1
    for n in n_tot:
        D = _lcm(D, n)
    sum_b = 0
    s_d = 0
    for w, a, n_w in zip(p.workers, assign, n_tot):
        b_w = sum(w.beta[g][c] for g, c in enumerate(a)) + switch_cost * switch_total(a)
        u_w = sum(w.n_kernels[g] * p.configs[c] for g, c in enumerate(a))
        sum_b += b_w
        s_d += u_w * (D // n_w)
    excess = max(0, s_d - T * D)
    if p.overlap_mode == OVERLAP_EXCESS:
        num = sum_b * (T * D + excess)
    elif p.overlap_mode == OVERLAP_LITERAL:
        num = sum_b * (T * D + s_d)
    else:
        idx = min(len(p.alpha_ppm) - 1, excess // (D * p.granule))
        num = sum_b * (10 ** 6 + p.alpha_ppm[idx])
    return num, s_d, switches


def solve_exhaustive(p) -> Tuple[List[List[int]], int, List[int]]:
    """Enumerate every assignment; return (assignment, objective numerator, switches per worker)."""
    n_c = len(p.configs)
    sizes = [len(w.n_kernels) for w in p.workers]
    total_units = sum(sizes)
    best_key = None
    best = None
    for flat in itertools.product(range(n_c), repeat=total_units):
        assign, pos = [], 0
        for g in sizes:
            assign.append(flat[pos:pos + g])
            pos += g
        r = evaluate(p, assign)
        if r is None:
            continue
        key = (r[0], r[1], flat)
        if best_key is None or key < best_key:
            best_key, best = key, (assign, r)
    if best is None:
        raise ValueError("no feasible assignment")
    assign, (num, _s, sw) = best
    return [list(a) for a in assign], num, sw


# ---- the two comparison policies of Sec. IV ("Spatial Partitioning Scenarios") --------------------------------------
def model_wise(p, slo_num: int = 3, slo_den: int = 1) -> Tuple[List[List[int]], List[int]]:
    """Model-Wise: each worker keeps ONE configuration for its whole request: the fewest CUs whose request latency
    (sum of its units' profiled latencies) is at most slo_num/slo_den times the latency on the largest configuration
    (Sec. II-A: QoS = 3x the solo latency).  Returns (assignment, switches per worker = 0)."""
    assign = []
    last = len(p.configs) - 1
    for w in p.workers:
        total = [sum(row[c] for row in w.beta) for c in range(len(p.configs))]
        ok = [c for c in range(len(p.configs)) if total[c] * slo_den <= total[last] * slo_num]
        assign.append([min(ok)] * len(w.beta))
    return assign, [0] * len(p.workers)


def kernel_wise(p, tol_pct: int = 5) -> Tuple[List[List[int]], List[int]]:
    """KW-Prealloc: each unit at its own minimum-CU threshold (Sec. III-B, "Minimum CU Threshold Profiling": the fewest
    CUs without noticeable slowdown; reading: 100*beta[c] <= (100+tol_pct)*beta[largest]).  Returns (assignment,
    switches per worker: positions where consecutive units differ, the KW-Prealloc column of Table I)."""
    assign = []
    last = len(p.configs) - 1
    for w in p.workers:
        a = []
        for row in w.beta:
            ok = [c for c in range(len(p.configs)) if 100 * row[c] <= (100 + tol_pct) * row[last]]
            a.append(min(ok))
        assign.append(a)
    return assign, [switch_total(a) for a in assign]
