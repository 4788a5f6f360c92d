"""GPU tests of the stream pool and the executor: CU masks, group -> stream tables, cross-stream
ordering, co-located models on concurrent worker threads, error paths."""
import threading

import numpy as np
import pytest

import workloads as wl
import paper_2506_12598_amd as ec
from oracle import forward as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import GpuModel, dev_input, rel_to_range, shared_pool  # noqa: E402


def test_pool_reports_streams_and_cu_counts():
    pool = shared_pool()
    assert pool.device_cus() == 256
    for mid, n in enumerate([256, 32, 64, 128, 192, 256]):
        s, n_cu = pool.stream(mid)
        assert n_cu == n and s
    with pytest.raises(ec.EclipError) as e:
        pool.stream(99)
    assert e.value.status == ec.EINVAL


def test_mask_bit_beyond_device_is_rejected():
    with pytest.raises(ec.EclipError) as e:
        ec.Pool([([0, 0, 0, 0, 0, 0, 0, 0, 1], -1)])
    assert e.value.status == ec.EINVAL and "device has" in e.value.message


def test_mask_that_empties_an_xcd_is_rejected():
    # all 32 CUs of XCD 0 and nothing elsewhere: the runtime cannot take such a queue mask
    with pytest.raises(ec.EclipError) as e:
        ec.Pool([(ec.words_of_bits([8 * j for j in range(32)], 8), -1)])
    assert e.value.status == ec.EINVAL and "XCD" in e.value.message


def test_masked_streams_confine_workgroups():
    pool = shared_pool()
    full = pool.probe(0, 2048)
    n_full = len(set(full.tolist()))
    assert n_full == 256, f"unmasked stream reached {n_full} distinct CUs"
    for mid, n in [(1, 32), (2, 64), (3, 128), (4, 192)]:
        ids = pool.probe(mid, 2048)
        assert len(set(ids.tolist())) == n, f"mask of {n} CUs ran on {len(set(ids.tolist()))} CUs"


def test_independent_layers_share_a_launch():
    """The projection shortcut and the first convolution of a residual block read the same tensor and do not depend on
    each other: the executor sends such a pair to the GPU as one launch; the global average pool and the classifier
    share one too, and the stem reads the caller's NCHW tensor itself instead of a channels-last copy made by a kernel of
    its own.  Same logits (within accumulation noise), five kernels fewer per ResNet-18 request; ECLIP_NO_PAIRS=1 turns
    the three fusions off."""
    import os
    m = wl.resnet(18, seed=1, hw=64)
    x = wl.make_input(m, 2)
    exp = orc.run_model(m, x)
    g = GpuModel(m, max_batch=2)
    try:
        got, (_, n_fused, _) = g.run(x, table=[0, 0, 0, 0], timing=True)
        os.environ["ECLIP_NO_PAIRS"] = "1"
        try:
            ref, (_, n_plain, _) = g.run(x, table=[0, 0, 0, 0], timing=True)
        finally:
            os.environ.pop("ECLIP_NO_PAIRS", None)
    finally:
        g.free()
    assert n_plain == 24 and n_fused == 19
    assert rel_to_range(got, exp) <= 2e-2 and rel_to_range(ref, exp) <= 2e-2
    assert np.abs(got - ref).max() <= 4e-3 * (exp.max() - exp.min())


def test_every_mask_and_table_gives_identical_logits():
    # the result must not depend on the CU share or on where group boundaries switch streams
    m = wl.resnet(18, seed=1, hw=64)
    x = wl.make_input(m, 1)
    g = GpuModel(m)
    try:
        ref = g.run(x, table=[0, 0, 0, 0])
        exp = orc.run_model(m, x)
        assert rel_to_range(ref, exp) <= 2e-2
        for table in ([1, 1, 1, 1], [5, 5, 5, 5], [1, 2, 3, 4], [4, 1, 4, 1], [0, 3, 3, 0], [2, 2, 5, 5]):
            got, (ns, n_k, n_sw) = g.run(x, table=table, timing=True)
            assert n_sw == sum(1 for i in range(1, 4) if table[i] != table[i - 1]) == g.h.switches()
            # 23 layers + the input re-layout; up to 3 pairs of independent convolutions share a launch, pool + classifier
            # too, and the stem may take over the re-layout
            assert 19 <= n_k <= 26 and ns > 0
            # split-K slice counts depend on the CU count, so sums may be associated differently:
            # compare within float32 accumulation noise of the 16-bit outputs
            assert rel_to_range(got, exp) <= 2e-2
            assert np.abs(got - ref).max() <= 2e-2 * (exp.max() - exp.min())
    finally:
        g.free()


def test_same_table_is_bit_reproducible():
    m = wl.resnet(18, seed=2, hw=64)
    x = wl.make_input(m, 1)
    g = GpuModel(m)
    try:
        a = g.run(x, table=[1, 3, 2, 5])
        for _ in range(5):
            assert np.array_equal(g.run(x, table=[1, 3, 2, 5]), a)
    finally:
        g.free()


def test_requests_of_one_model_run_in_order_and_inflight_limit():
    m = wl.resnet(18, seed=1, hw=64)
    g = GpuModel(m, max_inflight=3)
    try:
        g.h.alloc_set([1, 2, 1, 2])
        xs = [wl.make_input(m, 1, seed=100 + i) for i in range(3)]
        d_in = [dev_input(m, x) for x in xs]
        outs = [torch.zeros(m.out_shape(1), dtype=torch.float32, device="cuda") for _ in xs]
        reqs = [g.h.submit(d_in[i].data_ptr(), outs[i].data_ptr(), 1) for i in range(3)]
        with pytest.raises(ec.EclipError) as e:
            g.h.submit(d_in[0].data_ptr(), outs[0].data_ptr(), 1)
        assert e.value.status == ec.ELIMIT
        with pytest.raises(ec.EclipError) as e:
            g.h.free()
        assert e.value.status == ec.ESTATE
        for r in reversed(reqs):        # waiting out of order is allowed
            r.wait()
        for x, o in zip(xs, outs):
            exp = orc.run_model(m, x)
            assert rel_to_range(o.cpu().numpy().astype(np.float64), exp) <= 2e-2
        with pytest.raises(ec.EclipError) as e:
            reqs[0].wait()
        assert e.value.status == ec.ESTATE
    finally:
        g.free()


def test_submit_errors():
    m = wl.tiny_cnn()
    pool = shared_pool()
    h = ec.Model(pool, m, wl.to_storage(m.weights, m.dtype), max_batch=2)
    try:
        x = dev_input(m, wl.make_input(m, 1))
        out = torch.zeros((1, 10), dtype=torch.float32, device="cuda")
        with pytest.raises(ec.EclipError) as e:
            h.submit(x.data_ptr(), out.data_ptr(), 1)
        assert e.value.status == ec.ESTATE
        with pytest.raises(ec.EclipError) as e:
            h.alloc_set([0, 0])
        assert e.value.status == ec.EINVAL
        with pytest.raises(ec.EclipError) as e:
            h.alloc_set([77])
        assert e.value.status == ec.EINVAL
        h.alloc_set([0])
        with pytest.raises(ec.EclipError) as e:
            h.submit(x.data_ptr(), out.data_ptr(), 3)
        assert e.value.status == ec.EINVAL
        with pytest.raises(ec.EclipError) as e:
            pool.destroy()
        assert e.value.status == ec.ESTATE
    finally:
        h.free()


def test_two_colocated_models_on_worker_threads():
    # configuration 2 at reduced spatial size: two ResNet-18-style workers, each with its own masked streams
    pool = shared_pool()
    models = [wl.resnet(18, seed=1, hw=64), wl.resnet(18, seed=2, hw=64)]
    gms = [GpuModel(m, pool=pool) for m in models]
    tables = [[3, 3, 2, 1], [2, 3, 3, 4]]
    xs = [wl.make_input(m, 1) for m in models]
    exps = [orc.run_model(m, x) for m, x in zip(models, xs)]
    errs = [None, None]

    def worker(i):
        try:
            gms[i].h.alloc_set(tables[i])
            d_in = dev_input(models[i], xs[i])
            out = torch.zeros(models[i].out_shape(1), dtype=torch.float32, device="cuda")
            worst = 0.0
            for _ in range(30):
                gms[i].h.submit(d_in.data_ptr(), out.data_ptr(), 1).wait()
                worst = max(worst, rel_to_range(out.cpu().numpy().astype(np.float64), exps[i]))
            errs[i] = worst
        except Exception as ex:      # noqa: BLE001
            errs[i] = ex
    th = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    [t.start() for t in th]
    [t.join() for t in th]
    for g in gms:
        g.free()
    for e in errs:
        assert isinstance(e, float) and e <= 2e-2, e


def test_profile_group_and_allocator_end_to_end():
    m = wl.resnet(18, seed=1, hw=64)
    g = GpuModel(m)
    try:
        configs = [32, 64, 128, 192, 256]
        beta, nk = [], []
        for grp in range(m.n_groups):
            row = []
            for mid in range(1, 6):
                ns = g.h.profile_group(grp, mid, batch=1, iters=5)
                assert len(ns) == g.h.group_size(grp) and all(v > 0 for v in ns)
                row.append(sum(ns))
            beta.append(row)
            nk.append(g.h.group_size(grp))
        assign, obj, sw = ec.eclip_alloc_solve(256, configs, [nk, nk], [beta, beta], 14)
        assert len(assign) == 2 and all(0 <= c < 5 for a in assign for c in a) and obj > 0
        x = wl.make_input(m, 1)
        got = g.run(x, table=[c + 1 for c in assign[0]])
        assert rel_to_range(got, orc.run_model(m, x)) <= 2e-2
    finally:
        g.free()


def test_per_kernel_groups_with_switching_tables_match_the_oracle():
    """Every kernel is a kernel group of its own (the unit of the paper's model, Sec. III-B): per-kernel latency tables
    are profiled on the masked streams, the optimizer (switch budget 14 per request), the per-kernel minimum-CU policy
    (KW-Prealloc) and the one-configuration policy (Model-Wise) each give a table, each table is installed and served
    through eclip_submit, and the output must match the oracle whatever the table.  The switch count of a request is the
    number of group boundaries that change stream."""
    import dataclasses
    configs = [32, 64, 128, 192, 256]
    for base, batch in ((wl.resnet(18, seed=1, hw=64), 2), (wl.bert(2, 128, 4, 256, 48, vocab=500, seed=4), 1)):
        m = dataclasses.replace(base, group_of_layer=list(range(len(base.layers))), n_groups=len(base.layers))
        x = wl.make_input(m, batch)
        exp = orc.run_model(m, x)
        g = GpuModel(m, max_batch=batch)
        try:
            beta = []
            for k in range(m.n_groups):
                assert g.h.group_size(k) == 1
                beta.append([g.h.profile_group(k, mid, batch=batch, iters=3)[0] for mid in range(1, 6)])
            ones = [1] * m.n_groups
            tables = []
            a, obj, sw = ec.eclip_alloc_solve(256, configs, [ones, ones], [beta, beta], 14)
            assert obj > 0 and all(s <= 14 for s in sw)
            tables.append(("optimizer, switchMax 14", a[0], sw[0]))
            a, sw = ec.eclip_alloc_kernel_wise(configs, [beta], 5)
            tables.append(("kernel-wise", a[0], sw[0]))
            a, sw = ec.eclip_alloc_model_wise(configs, [beta], 3, 1)
            assert sw == [0] and len(set(a[0])) == 1
            tables.append(("model-wise", a[0], 0))
            # a table that switches at every boundary, whatever the profile said
            tables.append(("alternating", [k % 2 * 3 for k in range(m.n_groups)], m.n_groups - 1))
            for name, assign, n_sw in tables:
                got, (_, n_k, got_sw) = g.run(x, table=[c + 1 for c in assign], timing=True)
                assert got_sw == n_sw == g.h.switches(), name
                assert n_k >= m.n_groups, name                 # no launch is shared across kernel groups
                assert rel_to_range(got, exp) <= 2e-2, name
        finally:
            g.free()


def test_served_group_profile_counts_the_launches_that_are_served():
    m = wl.resnet(18, seed=1, hw=64)
    g = GpuModel(m)
    try:
        x = wl.make_input(m, 1)
        _, (_, n_served, _) = g.run(x, table=[2, 2, 2, 2], timing=True)
        total = 0
        for grp in range(m.n_groups):
            ns, n = g.h.profile_group_served(grp, 2, batch=1, iters=3)
            per_layer = g.h.profile_group(grp, 2, batch=1, iters=3)
            assert ns > 0 and 1 <= n <= g.h.group_size(grp) + (1 if grp == 0 else 0)
            assert ns < 3 * sum(per_layer) + 50_000            # same order as the per-layer figures
            total += n
        assert total == n_served                               # the profiler walks the launch sequence of eclip_submit
    finally:
        g.free()


def test_replayed_graphs_stay_on_the_streams_cus_and_give_the_same_bits():
    """eclip_model_graphs: a request is captured once per (buffers, batch, table) as one HIP graph per run of kernel groups
    on the same stream and replayed afterwards.  A graph replayed on a CU-masked stream must stay on that stream's CUs;
    the replayed request must give the bits of the launched one, on every replay, across table changes, with the program's
    own eager work in between (the layout kernels of the input copies, synchronisations)."""
    pool = shared_pool()
    for mid, n in [(1, 32), (2, 64), (4, 192)]:
        ids = pool.probe_graph(mid, 2048)
        assert len(set(ids.tolist())) == n and set(ids.tolist()) == set(pool.probe(mid, 2048).tolist())
    m = wl.resnet(18, seed=1, hw=64)
    g = GpuModel(m, max_batch=2)
    try:
        xs = [wl.make_input(m, 2, seed=50 + i) for i in range(3)]
        tables = ([1, 1, 1, 1], [1, 3, 3, 2], [4, 1, 4, 1])
        ref = {(ti, xi): g.run(x, table=list(t)) for ti, t in enumerate(tables) for xi, x in enumerate(xs)}
        g.h.graphs(True)
        d_in = [dev_input(m, x) for x in xs]
        outs = [torch.zeros(m.out_shape(2), dtype=torch.float32, device="cuda") for _ in xs]
        for rep in range(3):                                    # replays after the first, with eager work between them
            for ti, t in enumerate(tables):
                g.h.alloc_set(list(t))
                for xi in range(3):
                    outs[xi].zero_()
                    r = g.h.submit(d_in[xi].data_ptr(), outs[xi].data_ptr(), 2)
                    _, n_k, n_sw = r.wait(timing=True)
                    assert n_sw == sum(1 for i in range(1, 4) if t[i] != t[i - 1]) and n_k >= 19
                    torch.cuda.synchronize()
                    assert np.array_equal(outs[xi].cpu().numpy().astype(np.float64), ref[(ti, xi)]), (rep, ti, xi)
        # batch 1 through the same buffers is another captured request
        r = g.h.submit(d_in[0].data_ptr(), outs[0].data_ptr(), 1)
        r.wait()
        assert np.array_equal(outs[0][:1].cpu().numpy().astype(np.float64), ref[(2, 0)][:1])
        g.h.graphs(False)
        assert np.array_equal(g.run(xs[1], table=[1, 1, 1, 1]), ref[(0, 1)])
    finally:
        g.free()


def test_measured_plan_selection_keeps_the_results():
    """eclip_model_tune times every candidate plan of every GEMM problem on a stream and remembers the fastest for that CU
    count; the logits must stay within tolerance of the oracle (another tile only reassociates fp32 sums), the same table
    must stay bit-reproducible, and untuned CU counts keep working."""
    for m, batch in ((wl.resnet(50, seed=3, hw=64), 2), (wl.bert(2, 256, 4, 1024, 96, vocab=500, seed=4), 2)):
        x = wl.make_input(m, batch)
        exp = orc.run_model(m, x)
        g = GpuModel(m, max_batch=batch)
        try:
            before = g.run(x, table=[2] * m.n_groups)
            n = g.h.tune(2, batch=batch, iters=1)
            assert n >= 3
            assert g.h.tune(2, batch=batch, iters=1) == 0         # every problem of this CU count is known now
            after = g.run(x, table=[2] * m.n_groups)
            assert np.array_equal(after, g.run(x, table=[2] * m.n_groups))
            other = g.run(x, table=[4] * m.n_groups)              # a CU count that was never tuned
            for got in (before, after, other):
                assert rel_to_range(got, exp) <= 2e-2
            info = g.h.kernel_info(len(m.layers) - 1, 2, batch)
            assert info["kernel"] in ("conv_wsk_kernel", "conv_gemm_kernel", "gap_kernel", "row_kernel")
        finally:
            g.free()


def test_switch_overhead_bench_runs():
    same, pooled, create = shared_pool().bench_switch(1, 2, 200)
    assert same > 0 and pooled > 0 and create > 0


def test_wait_timeout_then_success():
    m = wl.resnet(18, seed=1, hw=64)
    g = GpuModel(m)
    try:
        d_in = dev_input(m, wl.make_input(m, 1))
        out = torch.zeros(m.out_shape(1), dtype=torch.float32, device="cuda")
        r = g.h.submit(d_in.data_ptr(), out.data_ptr(), 1)
        try:
            r.wait(timeout_ns=1)          # may or may not have finished within a nanosecond
        except ec.EclipError as e:
            assert e.status == ec.ETIMEOUT
            r.wait()
    finally:
        g.free()


def test_pipes_rebind_and_stream_chain():
    pool = shared_pool()
    assert pool.pipe(0) == 2 ** 32 - 1                      # unmasked stream: one of the runtime's shared queues
    assert [pool.pipe(i) for i in range(1, 6)] == [0, 1, 2, 3, 0]
    t1 = pool.bench_streams([1], 200)
    t4 = pool.bench_streams([1, 2, 3, 4], 200)
    assert t1 > 0 and t4 > 0
    # a model moves to a second pool and still computes the same logits
    m = wl.resnet(18, seed=1, hw=64)
    x = wl.make_input(m, 1)
    g = GpuModel(m)
    try:
        ref = g.run(x, table=[1, 1, 2, 2])
        small = ec.Pool([(ec.eclip_mask_layout(256, 32, 2, 0, 4), 0), (ec.eclip_mask_layout(256, 32, 2, 0, 2), 0)])
        g.h.rebind(small)
        with pytest.raises(ec.EclipError) as e:
            g.run(x)                                         # the table was cleared by the move
        assert e.value.status == ec.ESTATE
        got = g.run(x, table=[0, 0, 1, 1])
        assert np.abs(got - ref).max() <= 2e-2 * (ref.max() - ref.min())
        g.h.rebind(pool)
        small.destroy()
        g.h.alloc_set([0, 0, 0, 0])
    finally:
        g.free()
