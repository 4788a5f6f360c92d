"""Pins for the allocation oracle (exhaustive search over the paper's Sec. III-B model)."""
import os

import pytest

import workloads as wl
from oracle import alloc as oa

GOLD = os.path.join(os.path.dirname(__file__), "golden")
CFG = [15, 30, 45, 60]


def worked_problem(mode):
    a = wl.Worker([1, 1], [[100, 60, 50, 45], [80, 70, 65, 64]])
    b = wl.Worker([1], [[200, 110, 80, 60]])
    return wl.AllocProblem(60, CFG, [a, b], 1, mode)


def read_gold():
    ev, best = [], []
    for line in open(os.path.join(GOLD, "alloc_worked_example.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        mode = {"EXCESS": oa.OVERLAP_EXCESS, "LITERAL": oa.OVERLAP_LITERAL}[t[1]]
        (ev if t[0] == "eval" else best).append((mode, [int(v) for v in t[2:]]))
    return ev, best


def test_hand_worked_example_evaluations():
    ev, _ = read_gold()
    assert len(ev) >= 10
    for mode, (ca0, ca1, cb, _sumb, s_d, num) in ev:
        p = worked_problem(mode)
        r = oa.evaluate(p, [[CFG.index(ca0), CFG.index(ca1)], [CFG.index(cb)]])
        assert r is not None and r[0] == num and r[1] == s_d


def test_hand_worked_example_optimum_and_tie_break():
    _, best = read_gold()
    for mode, (i0, i1, i2, num, s0, s1) in best:
        assign, obj, sw = oa.solve_exhaustive(worked_problem(mode))
        assert assign == [[i0, i1], [i2]] and obj == num and sw == [s0, s1]


def test_calibration_two_identical_kernels_take_twice_as_long():
    # Sec. III-B calibrates alpha on one observation: a kernel co-run with a copy of itself on the same CUs needs 2x its solo time -> alpha = 1.
    beta = 1000
    p = wl.AllocProblem(60, [60], [wl.Worker([1], [[beta]]), wl.Worker([1], [[beta]])], 0, oa.OVERLAP_EXCESS)
    _, num, _ = oa.solve_exhaustive(p)
    assert num == (2 * beta * 2) * 60          # J = 2*beta*(1+1), scaled by T*D = 60
    # a lone worker on the whole GPU is not slowed down under EXCESS ...
    solo = wl.AllocProblem(60, [60], [wl.Worker([1], [[beta]])], 0, oa.OVERLAP_EXCESS)
    assert oa.solve_exhaustive(solo)[1] == beta * 60
    # ... but is (alpha = 1) under the formula as printed, which is why EXCESS is the default reading
    solo.overlap_mode = oa.OVERLAP_LITERAL
    assert oa.solve_exhaustive(solo)[1] == 2 * beta * 60


def test_switch_count_identity_onehot_form():
    import random
    r = random.Random(5)
    for _ in range(200):
        n, k = r.randint(1, 12), r.randint(1, 5)
        v = [r.randrange(k) for _ in range(n)]
        assert oa.switch_total(v) == oa.switch_total_onehot(v, k)
    assert oa.switch_total([0, 0, 1, 1, 0]) == 2 and oa.switch_total([3]) == 0


def test_single_worker_takes_per_unit_argmin_when_budget_allows():
    for seed in range(20):
        p = wl.random_problem(seed, 1, [4], [32, 64, 128, 192, 256], 256, switch_max=3, shape="random")
        assign, num, sw = oa.solve_exhaustive(p)
        w = p.workers[0]
        for g, c in enumerate(assign[0]):
            assert w.beta[g][c] == min(w.beta[g])
        n = sum(w.n_kernels)
        assert num == sum(min(r) for r in w.beta) * 256 * n      # alpha = 0, scaled by T*D


def test_flat_tables_choose_fewest_cus():
    p = wl.random_problem(3, 2, [3, 2], [32, 64, 128], 128, switch_max=2, shape="flat")
    assign, _, sw = oa.solve_exhaustive(p)
    assert assign == [[0, 0, 0], [0, 0]] and sw == [0, 0]


def test_zero_budget_means_one_config_per_worker():
    for seed in range(10):
        p = wl.random_problem(100 + seed, 2, [3, 3], [15, 30, 45, 60], 60, switch_max=0)
        assign, num, sw = oa.solve_exhaustive(p)
        assert sw == [0, 0] and all(len(set(a)) == 1 for a in assign)
        # |C|^W candidates evaluated directly
        cands = [oa.evaluate(p, [[a] * 3, [b] * 3])[0] for a in range(4) for b in range(4)]
        assert num == min(cands)


def test_objective_monotone_in_switch_budget_and_table_i_bound():
    for seed in range(10):
        prev = None
        for sm in range(0, 4):
            p = wl.random_problem(200 + seed, 2, [4, 2], [15, 30, 45, 60], 60, switch_max=sm)
            assign, num, sw = oa.solve_exhaustive(p)
            assert all(s <= sm for s in sw)
            assert all(0 <= c < 4 for a in assign for c in a)           # one valid config per unit
            if prev is not None:
                assert num <= prev
            prev = num


def test_infeasible_assignment_is_rejected():
    p = worked_problem(oa.OVERLAP_EXCESS)
    p.switch_max = 0
    assert oa.evaluate(p, [[0, 1], [0]]) is None


def test_table_mode_uses_excess_granules():
    a = wl.Worker([1], [[100, 50]])
    b = wl.Worker([1], [[100, 50]])
    p = wl.AllocProblem(64, [32, 64], [a, b], 0, oa.OVERLAP_TABLE, alpha_ppm=[0, 300000, 900000], granule=32)
    # (64,64): excess 64 -> granule 2 -> 100*(1.9) = 190 ; (32,64): excess 32 -> 150*1.3 = 195 ; (32,32): 200
    assign, num, _ = oa.solve_exhaustive(p)
    assert assign == [[1], [1]] and num == 100 * 1_900_000


def test_extension_max_configs_and_switch_cost_hand_checked():
    # worked instance again (EXCESS): optimum without limits is (30,30 | 30) = 28800 with no switch at all, so neither
    # extension changes it ...
    p = worked_problem(oa.OVERLAP_EXCESS)
    p.max_configs, p.switch_cost = 1, 1000
    assert oa.solve_exhaustive(p)[0] == [[1, 1], [1]]
    # ... LITERAL optimum (30,15 | 45) = 220 * 255 = 56100 uses one switch: a switch cost of 10 ns makes it
    # (220 + 10) * 255 = 58650, worse than the best switch-free choice:
    #   (30,30 | 45): 210 * (120 + 150) = 56700 ; (30,30 | 30): 240 * 240 = 57600 ; (15,15 | 45): 260 * 240 = 62400
    #   (45,45 | 60): 175 * (120 + 210) = 57750 ; (30,30 | 60): 190 * 300 = 57000 ; (45,45 | 45): 195 * 300 = 58500
    p = worked_problem(oa.OVERLAP_LITERAL)
    p.switch_cost = 10
    assert oa.evaluate(p, [[1, 0], [2]])[0] == 58650
    assign, num, sw = oa.solve_exhaustive(p)
    assert (assign, num, sw) == ([[1, 1], [2]], 56700, [0, 0])
    # the same answer is forced by allowing one configuration per worker
    p = worked_problem(oa.OVERLAP_LITERAL)
    p.max_configs = 1
    assert oa.solve_exhaustive(p)[0] == [[1, 1], [2]]
    assert oa.evaluate(p, [[1, 0], [2]]) is None


# ---------------- the comparison policies of Sec. IV: Model-Wise and KW-Prealloc ----------------
def _worked_instance():
    return wl.AllocProblem(60, [15, 30, 45, 60], [wl.Worker([1, 1], [[100, 60, 50, 45], [80, 70, 65, 64]]),
                                                   wl.Worker([1], [[200, 110, 80, 60]])], 1)


def _policy_rows(kind):
    path = os.path.join(os.path.dirname(__file__), "golden", "policies_worked_example.txt")
    return [[int(v) for v in ln.split()[1:]] for ln in open(path) if ln.startswith(kind + " ")]


def test_model_wise_and_kernel_wise_hand_worked_golden():
    p = _worked_instance()
    rows = _policy_rows("model_wise")
    assert len(rows) == 3
    for num, den, a, b in rows:
        assign, sw = oa.model_wise(p, num, den)
        assert assign == [[a, a], [b]] and sw == [0, 0]
    rows = _policy_rows("kernel_wise")
    assert len(rows) == 3
    for tol, a0, a1, b, sa, sb in rows:
        assign, sw = oa.kernel_wise(p, tol)
        assert assign == [[a0, a1], [b]] and sw == [sa, sb]


def test_policy_ties_flat_tables_and_monotonicity():
    # a table that does not depend on the CU count: every configuration qualifies, the fewest CUs win
    flat = wl.AllocProblem(60, [15, 30, 45, 60], [wl.Worker([1, 1, 1], [[70] * 4, [9] * 4, [123] * 4])], 0)
    assert oa.model_wise(flat, 1, 1) == ([[0, 0, 0]], [0])
    assert oa.kernel_wise(flat, 0) == ([[0, 0, 0]], [0])
    # equality counts as meeting the threshold (the inequalities are not strict)
    eq = wl.AllocProblem(60, [15, 30, 60], [wl.Worker([1], [[210, 105, 100]])], 0)
    assert oa.kernel_wise(eq, 5)[0] == [[1]] and oa.kernel_wise(eq, 4)[0] == [[2]]
    assert oa.model_wise(eq, 21, 10)[0] == [[0]] and oa.model_wise(eq, 2, 1)[0] == [[1]]
    for seed in range(20):
        p = wl.random_problem(seed, 2, [4, 3], [32, 64, 128, 192, 256], 256, 14)
        last = len(p.configs) - 1
        prev_mw, prev_kw = None, None
        for tol in (0, 5, 20, 100, 1000):
            kw, sw = oa.kernel_wise(p, tol)
            mw, _ = oa.model_wise(p, 100 + tol, 100)
            # the chosen configuration meets the rule and the next smaller one does not
            for w, a in zip(p.workers, kw):
                for row, c in zip(w.beta, a):
                    assert 100 * row[c] <= (100 + tol) * row[last]
                    assert all(100 * row[d] > (100 + tol) * row[last] for d in range(c))
            assert sw == [oa.switch_total(a) for a in kw]
            assert all(len(set(a)) == 1 for a in mw)
            # a looser target never asks for more CUs
            if prev_kw is not None:
                assert all(c <= d for a, b in zip(kw, prev_kw) for c, d in zip(a, b))
                assert all(a[0] <= b[0] for a, b in zip(mw, prev_mw))
            prev_mw, prev_kw = mw, kw
        # a single-unit worker: both policies coincide at the same tolerance
        one = wl.AllocProblem(256, p.configs, [wl.Worker([1], [p.workers[0].beta[0]])], 0)
        assert oa.model_wise(one, 105, 100)[0] == oa.kernel_wise(one, 5)[0]
