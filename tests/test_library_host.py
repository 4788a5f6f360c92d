"""Host-side tests of libeclip that need no GPU: exported symbols, the exact allocation solver against
the exhaustive-search oracle (bit-exact decisions), the mask layout against the paper's worked example,
descriptor validation and error paths."""
import os
import re

import pytest

import workloads as wl
import paper_2506_12598_amd as ec
from oracle import alloc as oa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "eclip.h")).read()
    declared = set(re.findall(r"\b(eclip_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(ec.lib, name), f"{name} declared in eclip.h but not exported"
    assert declared == set(ec.EXPORTS), "binding and header disagree on the entry points"


def solve_lib(p):
    return ec.eclip_alloc_solve(p.total_cus, p.configs, [w.n_kernels for w in p.workers], [w.beta for w in p.workers],
                                p.switch_max, p.overlap_mode, p.alpha_ppm, p.granule, p.max_configs, p.switch_cost, p.max_configs_w)


CASES = []
for seed in range(12):
    for mode in (oa.OVERLAP_EXCESS, oa.OVERLAP_LITERAL, oa.OVERLAP_TABLE):
        CASES.append((seed, 2, [3, 3], [32, 64, 128, 192, 256], 256, 1 + seed % 2, mode, "scaling"))
        CASES.append((50 + seed, 3, [2, 2, 2], [15, 30, 45, 60], 60, seed % 3, mode, "random"))
        CASES.append((90 + seed, 2, [4, 2], [32, 64, 128], 128, 1, mode, "ties"))
        CASES.append((130 + seed, 1, [6], [16, 48, 96, 256], 256, 2, mode, "scaling"))
        CASES.append((170 + seed, 4, [1, 2, 1, 2], [64, 128, 256], 256, 1, mode, "scaling"))


@pytest.mark.parametrize("seed,nw,units,configs,total,sm,mode,shape", CASES)
def test_solver_matches_exhaustive_oracle_bit_exact(seed, nw, units, configs, total, sm, mode, shape):
    p = wl.random_problem(seed, nw, units, configs, total, sm, mode, shape)
    exp_assign, exp_obj, exp_sw = oa.solve_exhaustive(p)
    got_assign, got_obj, got_sw = solve_lib(p)
    assert got_assign == exp_assign
    assert got_obj == exp_obj
    assert got_sw == exp_sw


EXT_CASES = [(seed, mc, sc, mode) for seed in range(8) for mc, sc in ((1, 0), (2, 0), (0, 700), (2, 3000), (1, 50))
             for mode in (oa.OVERLAP_EXCESS, oa.OVERLAP_TABLE)]


@pytest.mark.parametrize("seed,max_configs,switch_cost,mode", EXT_CASES)
def test_solver_extensions_match_exhaustive_oracle_bit_exact(seed, max_configs, switch_cost, mode):
    for units, configs, total, sm, shape in (([3, 3], [32, 64, 128, 192, 256], 256, 2, "scaling"),
                                             ([2, 2, 2], [15, 30, 45, 60], 60, 1, "random"),
                                             ([4, 2], [32, 64, 128], 128, 3, "ties")):
        p = wl.random_problem(300 + seed, len(units), units, configs, total, sm, mode, shape)
        p.max_configs, p.switch_cost = max_configs, switch_cost
        exp = oa.solve_exhaustive(p)
        got = solve_lib(p)
        assert got[0] == exp[0] and got[1] == exp[1] and got[2] == exp[2]
        if max_configs:
            assert all(len(set(a)) <= max_configs for a in got[0])


def test_solver_hand_worked_example():
    a = wl.Worker([1, 1], [[100, 60, 50, 45], [80, 70, 65, 64]])
    b = wl.Worker([1], [[200, 110, 80, 60]])
    assign, obj, sw = solve_lib(wl.AllocProblem(60, [15, 30, 45, 60], [a, b], 1, oa.OVERLAP_EXCESS))
    assert (assign, obj, sw) == ([[1, 1], [1]], 28800, [0, 0])
    assign, obj, sw = solve_lib(wl.AllocProblem(60, [15, 30, 45, 60], [a, b], 1, oa.OVERLAP_LITERAL))
    assert (assign, obj, sw) == ([[1, 0], [2]], 56100, [1, 0])


def test_solver_scales_to_config_sized_instances_and_respects_budget():
    # four workers, 24 units each, five configurations: far beyond exhaustive search; check validity and
    # that the result is no worse than simple feasible assignments evaluated by the oracle
    p = wl.random_problem(7, 4, [24, 24, 7, 12], [32, 64, 128, 192, 256], 256, 14, oa.OVERLAP_EXCESS, max_kernels=9)
    assign, obj, sw = solve_lib(p)
    r = oa.evaluate(p, assign)
    assert r is not None and r[0] == obj and r[2] == sw and all(s <= 14 for s in sw)
    for c in range(5):
        uni = [[c] * len(w.n_kernels) for w in p.workers]
        assert obj <= oa.evaluate(p, uni)[0]


def test_solver_rejects_malformed_problems():
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_solve(256, [64, 32], [[1]], [[[5, 5]]], 1)
    assert e.value.status == ec.EINVAL and "increasing" in e.value.message
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_solve(256, [32, 64], [[0]], [[[5, 5]]], 1)
    assert e.value.status == ec.EINVAL
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_solve(256, [32, 64], [[1]], [[[5, 5]]], 1, ec.OVERLAP_TABLE, None, 1)
    assert e.value.status == ec.EINVAL
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_solve(256, [1, 256], [[4000] * 64], [[[5, 5]] * 64], 14)
    assert e.value.status == ec.ELIMIT


# ---- mask layout (Sec. III-A worked example) ------------------------------------------------------------
def test_mask_layout_reproduces_paper_example():
    gold = []
    for line in open(os.path.join(ROOT, "tests", "golden", "mask_layout_example.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            gold.append((int(t[0]), int(t[1]), [int(v) for v in t[2:]]))
    assert len(gold) == 6
    for worker, n_cus, ses in gold:
        words = ec.eclip_mask_layout(60, 15, 2, worker - 1, n_cus // 15)
        bits = ec.mask_bits(words)
        assert len(bits) == n_cus
        assert sorted({b // 15 + 1 for b in bits}) == ses
        for se in ses:          # whole shader engines only
            assert all((se - 1) * 15 + j in bits for j in range(15))


@pytest.mark.parametrize("total,granule,striped", [(60, 15, 0), (256, 32, 0), (256, 64, 8), (256, 32, 8), (60, 15, 1)])
def test_mask_layout_two_workers_overlap_only_in_the_excess(total, granule, striped):
    ng = total // granule
    for a in range(1, ng + 1):
        ma = set(ec.mask_bits(ec.eclip_mask_layout(total, granule, 2, 0, a, striped)))
        assert len(ma) == a * granule
        if a > 1:      # masks of one worker are nested
            assert set(ec.mask_bits(ec.eclip_mask_layout(total, granule, 2, 0, a - 1, striped))) < ma
        for b in range(1, ng + 1):
            mb = set(ec.mask_bits(ec.eclip_mask_layout(total, granule, 2, 1, b, striped)))
            assert len(ma & mb) == max(0, a + b - ng) * granule


def test_mask_layout_striped_granules_keep_every_xcd_populated():
    # MI355X: mask bit i lies in XCD i % 8 and shader engine (i / 8) % 4.  stripe = 8, granule = 64: one whole
    # shader engine of every XCD per granule
    for worker, se in ((0, 0), (1, 3)):
        bits = ec.mask_bits(ec.eclip_mask_layout(256, 64, 2, worker, 1, stripe=8))
        assert len(bits) == 64
        assert {b % 8 for b in bits} == set(range(8))
        assert {(b // 8) % 4 for b in bits} == {se}
    # stripe = 0, granule = 32: one CU of every shader engine of every XCD per granule
    bits = ec.mask_bits(ec.eclip_mask_layout(256, 32, 2, 0, 1))
    assert bits == list(range(32))
    bits = ec.mask_bits(ec.eclip_mask_layout(256, 32, 2, 1, 1))
    assert bits == list(range(224, 256))


def test_mask_layout_errors():
    for args in [(60, 16, 2, 0, 1), (60, 15, 2, 2, 1), (60, 15, 2, 0, 5), (60, 15, 2, 0, 0), (256, 32, 2, 0, 1, 5)]:
        with pytest.raises(ec.EclipError) as e:
            ec.eclip_mask_layout(*args)
        assert e.value.status == ec.EINVAL


# ---- descriptor validation and error paths that need no device -----------------------------------------
def load_expect(model, status, text=None, **kw):
    with pytest.raises(ec.EclipError) as e:
        ec.Model(None, model, wl.to_storage(model.weights, model.dtype), **kw)
    assert e.value.status == status, e.value
    if text:
        assert text in e.value.message, e.value.message


def test_valid_descriptors_pass_validation_and_stop_at_the_null_pool():
    for m in [wl.tiny_cnn(), wl.resnet(18, hw=64), wl.resnet(50, hw=64), wl.vgg16(hw=32, width=16, fc=64),
              wl.mobilenetv2(hw=64), wl.bert(2, 128, 4, 512, 48, vocab=1000)] + wl.config_models(5, small=True) + \
            wl.config_models(6, small=True):
        load_expect(m, ec.EINVAL, "pool is null")


def test_descriptor_errors_of_the_second_workload_family():
    m = wl.config_models(5, small=True)[1]                       # DenseNet-style
    i = next(k for k, L in enumerate(m.layers) if L.op == wl.OP_CONCAT)
    m.layers[i].c += 8
    load_expect(m, ec.EINVAL, "summed channel count")
    m = wl.config_models(5, small=True)[1]
    m.layers[i].in1 = -2
    load_expect(m, ec.EINVAL, "two inputs")
    m = wl.config_models(6, small=True)[1]                       # ShuffleNet-style
    i = next(k for k, L in enumerate(m.layers) if L.op == wl.OP_SHUFFLE)
    m.layers[i].groups = 7
    load_expect(m, ec.EINVAL, "SHUFFLE groups")
    m = wl.config_models(6, small=True)[0]                       # ResNeXt-style
    i = next(k for k, L in enumerate(m.layers) if L.op == wl.OP_CONV and 1 < L.groups < L.c)
    m.layers[i].groups = 5
    load_expect(m, ec.EINVAL, "groups must divide")
    m = wl.single_layer("conv", wl.DT_F32, cin=16, cout=16, h=8, w=8, k=3, pad=1, groups=4)
    load_expect(m, ec.EINVAL, "16-bit model")


def test_descriptor_errors():
    m = wl.resnet(18, hw=64)
    m.group_of_layer[5] = 3
    load_expect(m, ec.EINVAL, "group_of_layer")
    m = wl.resnet(18, hw=64)
    m.layers[3].in0 = 7
    load_expect(m, ec.EINVAL, "not an earlier layer")
    m = wl.resnet(18, hw=64)
    m.layers[2].h += 1
    load_expect(m, ec.EINVAL, "expected")
    m = wl.resnet(18, hw=64)
    m.layers[4].w_off = len(m.weights) - 3
    load_expect(m, ec.EINVAL, "outside the weight blob")
    m = wl.resnet(18, hw=64)
    load_expect(m, ec.EINVAL, "max_batch", max_batch=0)
    m = wl.bert(1, 96, 2, 128, 16, vocab=100)        # head size 48
    load_expect(m, ec.EINVAL, "head size")
    m = wl.bert(1, 128, 4, 256, 16, vocab=100, dtype=wl.DT_F32)
    load_expect(m, ec.EINVAL, "16-bit")
    m = wl.single_layer("conv", cin=12, cout=16, h=8, w=8, k=3, pad=1)
    load_expect(m, ec.EINVAL, "pool is null")          # the 12-channel network input is padded by the loader
    m = wl.tiny_cnn(dtype=wl.DT_BF16)
    m.layers[0].c = 12                                 # a 12-channel tensor feeding a 16-bit conv
    m.layers[0].w_off = 0
    load_expect(m, ec.EINVAL)


def test_pool_errors_before_any_device_call():
    with pytest.raises(ec.EclipError) as e:
        ec.Pool([])
    assert e.value.status == ec.EINVAL
    with pytest.raises(ec.EclipError) as e:
        ec.Pool([([0, 0], -1)])
    assert e.value.status == ec.EINVAL and "no CU" in e.value.message
    with pytest.raises(ec.EclipError) as e:
        ec.Pool([([1], -1)] * 65)
    assert e.value.status == ec.ELIMIT


# ---------------- bench.py command line (no GPU) ------------------------------------------------------------------------
def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_traffic_file_is_tied_to_the_kernel_sources():
    """The counted HBM traffic in the bench line is only reported while the kernel sources are the ones the counters
    were taken on: the stored file carries their hash."""
    import json, os, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    h = bench.source_hash()
    assert len(h) == 64 and h == bench.source_hash()
    path = bench.traffic_path(1)
    if os.path.exists(path):
        d = json.load(open(path))
        assert set(("source_sha256", "kernels", "copy_scale_fetch", "copy_scale_write")) <= set(d)
        assert d["kernels"]["conv_wsk_kernel"]["fetch_bytes_per_launch"] > 0


# ---------------- Model-Wise and KW-Prealloc (Sec. IV scenarios) against the oracle's definitions ----------------
@pytest.mark.parametrize("seed", range(24))
def test_policies_match_the_oracle_bit_exact(seed):
    shape = ("scaling", "random", "ties", "flat")[seed % 4]
    units = [[5, 3], [2, 2, 2], [7], [1, 4, 2, 3]][seed % 4]
    configs = [[32, 64, 128, 192, 256], [15, 30, 45, 60], list(range(16, 257, 16)), [64, 128, 256]][(seed // 4) % 4]
    p = wl.random_problem(700 + seed, len(units), units, configs, configs[-1], 14, shape=shape)
    beta = [w.beta for w in p.workers]
    for num, den in ((3, 1), (3, 2), (1, 1), (105, 100)):
        assert ec.eclip_alloc_model_wise(p.configs, beta, num, den) == oa.model_wise(p, num, den)
    for tol in (0, 5, 12, 50, 400):
        got = ec.eclip_alloc_kernel_wise(p.configs, beta, tol)
        assert got == oa.kernel_wise(p, tol)
        assert all(s <= len(a) - 1 for a, s in zip(*got))


def test_policies_reject_malformed_input():
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_model_wise([32, 64], [[[5, 4]]], 1, 2)          # a target below the solo latency
    assert e.value.status == ec.EINVAL
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_kernel_wise([64, 32], [[[5, 4]]], 5)           # configurations not increasing
    assert e.value.status == ec.EINVAL
    with pytest.raises(ec.EclipError) as e:
        ec.eclip_alloc_kernel_wise([32, 64], [[]], 5)                 # a worker without units
    assert e.value.status == ec.EINVAL


@pytest.mark.parametrize("seed", range(10))
def test_per_worker_stream_limits_match_exhaustive_oracle_bit_exact(seed):
    """A global budget of 4 usable streams split unevenly over the workers: every composition is one solve with per-worker
    limits on the number of distinct configurations; each must equal exhaustive search, and the best of them is what a
    global limit would give."""
    units, configs = ([3, 2, 2], [32, 64, 128, 256]) if seed % 2 else ([3, 3], [32, 64, 128, 192, 256])
    p = wl.random_problem(900 + seed, len(units), units, configs, 256, 2, oa.OVERLAP_EXCESS, "scaling")
    p.switch_cost = 300 * (seed % 3)
    comps = [(2, 1, 1), (1, 2, 1), (1, 1, 2)] if len(units) == 3 else [(2, 2), (3, 1), (1, 3)]
    best = None
    for comp in comps:
        p.max_configs_w = list(comp)
        exp = oa.solve_exhaustive(p)
        got = solve_lib(p)
        assert got[0] == exp[0] and got[1] == exp[1] and got[2] == exp[2]
        assert all(len(set(a)) <= k for a, k in zip(got[0], comp))
        best = exp[1] if best is None else min(best, exp[1])
    # brute force over the union: total distinct (worker, configuration) pairs <= 4
    import itertools
    p.max_configs_w = None
    glob = None
    for flat in itertools.product(range(len(configs)), repeat=sum(units)):
        assign, pos = [], 0
        for g in units:
            assign.append(flat[pos:pos + g]); pos += g
        if sum(len(set(a)) for a in assign) > 4:
            continue
        r = oa.evaluate(p, assign)
        if r is not None:
            glob = r[0] if glob is None else min(glob, r[0])
    assert best == glob
