#!/usr/bin/env python3
"""Co-located inference benchmark on one MI355X.

Default workload (`--config 4`, the largest co-location mix and the one the headline metric is quoted on): three
BERT-large-style encoders (24 layers, hidden 1024, 16 heads, FFN 4096, seq 384, batch 4, bf16) and one
ResNet-152-style CNN (batch 8, bf16), each cut into kernel groups (3 encoder layers / a stage), served by one worker
thread per model on a pre-allocated pool of CU-masked streams (16..256 CUs in steps of 16 per worker) plus unmasked
streams.  The CU share of every group comes from the library's exact solver of the paper's allocation model
(Sec. III-B), fed with latency-vs-CU tables profiled here.  `--config 1|2|3` run the smaller mixes (2 x ResNet-18
batch 1; ResNet-50 + BERT-base; ResNet-50 + VGG-16 + MobileNetV2 + BERT-base with batch 1-8) through the same code.

One step = one request on every co-located model.  The timed region is exactly `--steps` steps under the ECLIP
policy with inputs resident in HBM; `value` is total inferences per second (a request of batch b counts b).
Around it, untimed: the same closed loop under the two unpartitioned policies, an open-loop Poisson run for
p50/p99 latency and inferences per joule, per-kernel HIP-event timings for the roofline entry, and the CPU
oracle timed on the host cores.

`--kernels` instead times single kernels at roofline shapes (operands far larger than the 256 MB last-level
cache) and prints a table; it is the command behind profiles/kernels_roofline_shapes.txt.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0
RIDGE = MFMA_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS       # FLOP per byte

WORKLOADS = {
    1: "2x ResNet-18-style bf16 batch 1 3x224x224, 4 kernel groups each",
    2: "ResNet-50-style bf16 batch 1 + BERT-base-style fp16 seq 128 batch 1, 4 kernel groups each",
    3: "ResNet-50 bf16 + VGG-16 bf16 + MobileNetV2 fp16 + BERT-base fp16, batch 1-8 uniform per request",
    4: "3x BERT-large-style bf16 seq 384 batch 4 + ResNet-152-style bf16 batch 8 (stress)",
    6: "second family: ALBERT-base-style fp16 seq 128 + DenseNet-121-style bf16, batch 1",
    7: "second family: ResNeXt-50-32x4d-style bf16 + ShuffleNet-g8-style bf16, batch 1",
    8: "VGG-16-style bf16 batch 8 + BERT-large-style bf16 seq 384 batch 4 (kernel groups with very different CU needs)",
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


# ---------------------------------------------------------------------------------------------------
# power sampling
# ---------------------------------------------------------------------------------------------------
class PowerSampler:
    """Samples board power (W) from the amdgpu hwmon node, falling back to `amd-smi metric -p --json`."""

    def __init__(self, hz: float = 20.0):
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")) or \
            sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        # the shader clock the GPU is running at: the level marked "*" in the amdgpu DPM table
        self.clk_paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.clocks = []
        self.dt = 1.0 / hz
        self.samples = []
        self.source = "hwmon" if self.paths else "amd-smi"
        self._stop = threading.Event()
        self._th = None

    def read(self):
        if self.paths:
            try:
                return int(open(self.paths[0]).read()) / 1e6
            except (OSError, ValueError):
                return None
        try:
            import subprocess
            out = subprocess.run(["amd-smi", "metric", "-p", "--json"], capture_output=True, text=True, timeout=5).stdout
            j = json.loads(out)
            node = j[0] if isinstance(j, list) else j.get("gpu_data", [j])[0]
            p = node["power"]["socket_power"]
            return float(p["value"] if isinstance(p, dict) else p)
        except Exception:   # noqa: BLE001
            return None

    def read_clock_mhz(self):
        try:
            cur = [l for l in open(self.clk_paths[0]).read().splitlines() if "*" in l][0]
            return float(cur.split(":")[1].lower().split("mhz")[0])
        except (OSError, ValueError, IndexError):
            return None

    def _run(self):
        while not self._stop.is_set():
            v = self.read()
            if v is not None:
                self.samples.append((time.perf_counter(), v))
            c = self.read_clock_mhz()
            if c is not None:
                self.clocks.append((time.perf_counter(), c))
            self._stop.wait(self.dt)

    def mean_clock_mhz(self, t0, t1):
        c = [v for t, v in self.clocks if t0 <= t <= t1]
        return float(np.mean(c)) if c else None

    def start(self):
        self.samples = []
        self.clocks = []
        self._stop.clear()
        self._th = threading.Thread(target=self._run, daemon=True)
        self._th.start()

    def stop(self):
        self._stop.set()
        self._th.join()

    def energy_j(self, t0, t1):
        s = [(t, p) for t, p in self.samples if t0 <= t <= t1]
        if len(s) < 2:
            return None
        t = np.array([a for a, _ in s]); p = np.array([b for _, b in s])
        e = float(np.trapezoid(p, t))
        return e * (t1 - t0) / (t[-1] - t[0])     # extend the covered span to the whole window


# ---------------------------------------------------------------------------------------------------
# workload
# ---------------------------------------------------------------------------------------------------
def gemm_work(model, batch):
    """(algorithmic bytes, flops) of every matrix-core conv/linear layer, None for other layers.  Bytes: input +
    weights + output (+ residual) once each, at the storage width; im2col duplication is not traffic."""
    import workloads as wl
    e = 4 if model.dtype == wl.DT_F32 else 2
    out = []
    for L in model.layers:
        if L.op not in (wl.OP_CONV, wl.OP_LINEAR) or L.groups != 1:
            out.append(None)
            continue
        if L.in0 == -1:
            cin, h, w, image = model.in_c, model.in_h, model.in_w, model.in_kind == wl.IN_IMAGE
        else:
            P = model.layers[L.in0]
            cin, h, w, image = P.c, P.h, P.w, P.kind == wl.KIND_IMAGE
        n_in = cin * h * w * batch
        n_out = L.c * L.h * L.w * batch
        taps = L.kh * L.kw if L.op == wl.OP_CONV else (h * w if image else 1)
        n_w = L.c * cin * taps
        flops = 2.0 * n_out * (n_w / L.c)
        out.append((float(e) * (n_in + n_w + n_out + (n_out if L.in1 != -2 else 0)), flops))
    return out


class Worker:
    """One model = one worker: holds the device buffers and runs closed-loop or scheduled requests."""

    def __init__(self, ec, torch, pool, model, index, depth, batches):
        import workloads as wl
        self.model, self.index, self.depth = model, index, depth
        self.batches = batches                       # per-request batch sizes, cycled
        self.max_batch = max(batches)
        self.h = ec.Model(pool, model, wl.to_storage(model.weights, model.dtype), max_batch=self.max_batch,
                          max_inflight=depth)
        x = wl.make_input(model, self.max_batch)
        self.x = x
        if model.in_kind == wl.IN_TOKENS:
            self.d_in = torch.from_numpy(x).cuda()
        else:
            s = wl.to_storage(x, model.dtype)
            self.d_in = torch.from_numpy(s.view(np.int16) if s.dtype == np.uint16 else s).cuda()
        self.d_out = [torch.zeros(model.out_shape(self.max_batch), dtype=torch.float32, device="cuda") for _ in range(depth)]
        self.served = 0
        self.error = None

    def closed_loop(self, n, barrier=None):
        """n requests, up to `depth` in flight; records the number of inferences served.  A failure is kept in
        self.error for the caller (run_closed raises it): a worker thread must never die silently."""
        self.error = None
        self.served = 0
        if barrier is not None:
            barrier.wait()
        q = []
        served = 0
        try:
            for i in range(n):
                if len(q) == self.depth:
                    q.pop(0).wait()
                b = self.batches[i % len(self.batches)]
                q.append(self.h.submit(self.d_in.data_ptr(), self.d_out[i % self.depth].data_ptr(), b))
                served += b
        except Exception as e:   # noqa: BLE001
            self.error = e
        for r in q:
            try:
                r.wait()
            except Exception as e:   # noqa: BLE001
                self.error = self.error or e
        self.served = served

    def open_loop(self, arrivals, t_start, lat_out):
        """Serve requests at their scheduled arrival times (seconds after t_start); latency = completion - arrival."""
        served = 0
        for i, a in enumerate(arrivals):
            now = time.perf_counter() - t_start
            if a > now:
                time.sleep(max(0.0, a - now - 50e-6))
                while time.perf_counter() - t_start < a:
                    pass
            b = self.batches[i % len(self.batches)]
            self.h.submit(self.d_in.data_ptr(), self.d_out[0].data_ptr(), b).wait()
            lat_out.append(time.perf_counter() - t_start - a)
            served += b
        self.served = served


def run_closed_for(workers, min_steps, seconds=1.0, warm_seconds=0.4):
    """Closed loop for measurements outside the timed region (calibration, trials between allocations): warms up until
    `warm_seconds` have passed (clocks and queues settle only after a few hundred milliseconds of load), then runs at
    least `min_steps` steps and at least about `seconds`.  Returns (elapsed, inferences served)."""
    t0 = time.perf_counter()
    chunk = max(2, min_steps // 5)
    while True:
        dt, _ = run_closed(workers, chunk)
        if time.perf_counter() - t0 >= warm_seconds:
            break
    n = int(min(50 * min_steps, max(min_steps, seconds / max(dt / chunk, 1e-6))))
    return run_closed(workers, n)


def run_closed(workers, steps):
    bar = threading.Barrier(len(workers) + 1)
    th = [threading.Thread(target=w.closed_loop, args=(steps, bar)) for w in workers]
    [t.start() for t in th]
    bar.wait()
    t0 = time.perf_counter()
    [t.join() for t in th]
    dt = time.perf_counter() - t0
    for w in workers:
        if w.error is not None:
            raise RuntimeError(f"worker {w.index} ({w.model.name}) failed: {w.error}")
    return dt, sum(w.served for w in workers)


# ---------------------------------------------------------------------------------------------------
# HBM traffic from hardware counters (two rocprofv3 --pmc runs of this file, reduced by --traffic-from)
# ---------------------------------------------------------------------------------------------------
CSRC = os.path.join(ROOT, "paper_2506_12598_amd", "csrc")
COPY_ROWS, COPY_WIDTH = 480000, 1024          # calibration copy: 2 x 983 MB read, 983 MB + 1966 MB written


def source_hash():
    import hashlib
    h = hashlib.sha256()
    for f in sorted(os.listdir(CSRC)):
        if f.endswith((".hip", ".h", ".cpp")):
            h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()


def measured_switch_cost_ns(pool, mask_a, mask_b):
    """Cost of one hop between two pooled masked streams beyond a launch on the same stream (Sec. III-A): median of five
    runs of eclip_bench_switch (a single run moves by a factor of ten with what else the queues are doing)."""
    d = []
    for _ in range(5):
        same_ns, pooled_ns, _ = pool.bench_switch(mask_a, mask_b, 1000, with_create=False)
        d.append(pooled_ns - same_ns)
    return max(0, int(sorted(d)[2]))


def traffic_path(cfg):
    return os.path.join(ROOT, "profiles", f"traffic_config{cfg}.json")


def pmc_copy(ec, torch):
    """One request of a two-layer element-wise model (plain copies of a known size): the calibration kernel for the
    FETCH_SIZE / WRITE_SIZE counters."""
    import workloads as wl
    import workloads.graphs as G
    bb = G._Builder("cp", wl.DT_BF16, 0, G.IN_SEQ, COPY_WIDTH, 1, COPY_ROWS)
    x = bb.eltwise(-1)
    bb.eltwise(x)
    m = bb.finish()
    pool = ec.Pool([(None, -1)])
    h = ec.Model(pool, m, wl.to_storage(m.weights, m.dtype), max_batch=1)
    h.alloc_set([0])
    d_in = torch.zeros((1, COPY_ROWS, COPY_WIDTH), dtype=torch.int16, device="cuda")
    d_out = torch.zeros((1, COPY_ROWS, COPY_WIDTH), dtype=torch.float32, device="cuda")
    h.submit(d_in.data_ptr(), d_out.data_ptr(), 1).wait()
    torch.cuda.synchronize()
    h.free(); pool.destroy()


def traffic_from(cfg, fetch_csv, write_csv, command):
    """Reduces the counter_collection CSVs of two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE; both of
    `bench.py --pmc-copy ...`) to HBM bytes per launch for every kernel function, scaled by what the same counter
    reads for the calibration copy, and stores them with a hash of the kernel sources."""
    import csv
    import re

    def reduce(path, counter):
        acc = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            m = re.search(r"(\w+)(<|\(|$)", r["Kernel_Name"].replace("void ", "").replace("eclip::(anonymous namespace)::", ""))
            name = m.group(1) if m else r["Kernel_Name"]
            a = acc.setdefault(name, [0.0, 0])
            a[0] += float(r["Counter_Value"]); a[1] += 1
        return acc

    n = COPY_ROWS * COPY_WIDTH * 2
    f, w = reduce(fetch_csv, "FETCH_SIZE"), reduce(write_csv, "WRITE_SIZE")
    assert f["eltwise_kernel"][1] == 2 and w["eltwise_kernel"][1] == 2, "expected the two calibration copies"
    scale_f = (2 * n) / (f["eltwise_kernel"][0] * 1024.0)          # counters are in KiB
    scale_w = (3 * n) / (w["eltwise_kernel"][0] * 1024.0)
    kernels = {}
    for k in f:
        if k in w and k != "eltwise_kernel":
            kernels[k] = {"dispatches": f[k][1], "fetch_bytes_per_launch": scale_f * 1024.0 * f[k][0] / f[k][1],
                          "write_bytes_per_launch": scale_w * 1024.0 * w[k][0] / w[k][1]}
    out = {"command": command, "counter_unit": "KiB", "copy_bytes_read": 2 * n, "copy_bytes_written": 3 * n,
           "copy_scale_fetch": scale_f, "copy_scale_write": scale_w, "kernels": kernels, "source_sha256": source_hash()}
    with open(traffic_path(cfg), "w") as fh:
        json.dump(out, fh, indent=1)
    print(json.dumps(out, indent=1))


def counters_from(csv_paths):
    """Reduces counter_collection CSVs of `rocprofv3 --pmc ...` runs to the mean of every counter per kernel (template
    arguments kept, so that tile shapes stay apart)."""
    import csv
    acc = {}
    for path in csv_paths:
        for r in csv.DictReader(open(path)):
            name = r["Kernel_Name"].replace("void ", "").replace("eclip::(anonymous namespace)::", "").replace("eclip::", "")
            name = name.split("(")[0][:96]
            a = acc.setdefault(name, {}).setdefault(r["Counter_Name"], [0.0, 0])
            a[0] += float(r["Counter_Value"]); a[1] += 1
    for name in sorted(acc):
        print(name)
        for c in sorted(acc[name]):
            v, n = acc[name][c]
            print(f"    {c:34s} dispatches {n:6d}  mean {v / n:.6g}")


def stats_from(trace_csv):
    """Reduces the kernel_trace CSV of `rocprofv3 --kernel-trace -- python3 bench.py ...` to a table per kernel function:
    all dispatches of the process, and those of the per-layer timing pass alone (between the last two probe_kernel
    dispatches, which bench.py launches around that pass).  In that pass every layer runs 8 times back to back on its
    worker's stream with nothing else on the GPU, which is what `roofline.avg_layer_us` times with HIP events.

    The profiler stamps a dispatch's start when its queue reaches it, which for a queue that has run dry is long
    before the host has even launched the kernel (one such row read 21 ms for a 5 us kernel), so the plain mean of
    End - Start is useless.  Durations are therefore reduced per (template instantiation, grid size), i.e. per tile shape
    and output size, to the median and to the mean over the dispatches within 8x that median (layers that share both
    differ in K by at most 4x here); the table pools them per function, weighting by calls."""
    import csv
    import re
    rd = csv.DictReader(open(trace_csv))
    col = {c.lower(): c for c in rd.fieldnames}
    c_name, c_st, c_en = col["kernel_name"], col["start_timestamp"], col["end_timestamp"]
    rows = []
    for r in rd:
        full = r[c_name].replace("void ", "").replace("eclip::(anonymous namespace)::", "").replace("eclip::", "")
        m = re.match(r"([\w:]+)", full)
        rows.append((int(r[c_st]), int(r[c_en]), m.group(1) if m else full, full.split("(")[0] + " grid " + r.get(col.get("grid_size_x", ""), "")))
    rows.sort()
    marks = [i for i, r in enumerate(rows) if r[2] == "probe_kernel"]

    def table(sel, title):
        by_inst = {}
        for i in sel:
            st, en, fn, inst = rows[i]
            by_inst.setdefault((fn, inst), []).append((en - st) / 1e3)
        acc = {}
        for (fn, inst), d in by_inst.items():
            d.sort()
            med = d[len(d) // 2]
            kept = [v for v in d if v <= 8.0 * med]
            a = acc.setdefault(fn, [0, 0, 0.0, 0.0])
            a[0] += len(d); a[1] += len(kept); a[2] += sum(kept); a[3] += med * len(d)
        tot = sum(a[2] for a in acc.values())
        print(f"# {title}")
        print(f"{'kernel':28s} {'calls':>9s} {'outliers':>9s} {'mean_us':>9s} {'median_us':>10s} {'share_%':>8s}")
        for fn, a in sorted(acc.items(), key=lambda kv: -kv[1][2]):
            print(f"{fn:28s} {a[0]:9d} {a[0] - a[1]:9d} {a[2] / a[1]:9.2f} {a[3] / a[0]:10.2f} {100.0 * a[2] / tot:8.2f}")

    # the marker kernel itself is left out: its dispatches follow idle queues, so their start stamps are the artefact above
    table([i for i in range(len(rows)) if rows[i][2] != "probe_kernel"],
          "all dispatches of the process (outliers: beyond 8x the median of their tile shape and grid, left out of the mean)")
    if len(marks) >= 2:
        table(range(marks[-2] + 1, marks[-1]), "per-layer timing pass (each layer 8 times back to back, alone on the GPU)")


# ---------------------------------------------------------------------------------------------------
# single kernels at roofline shapes
# ---------------------------------------------------------------------------------------------------
def kernels_mode(only=None, extra_gemms=None, tune=True, cus=256):
    import workloads as wl
    import workloads.graphs as G
    import paper_2506_12598_amd as ec
    # --cus N: the kernels run on a stream masked to N CUs (N / 8 in every XCD) and matrix-core rows are held against the
    # matrix peak scaled by N / 256
    sid = 0 if cus >= 256 else 1
    pool = ec.Pool([(None, -1)] + ([] if cus >= 256 else [(ec.eclip_mask_layout(256, 16, 1, 0, cus // 16), 0)]))
    mfma_peak = MFMA_PEAK_TFLOPS * min(cus, 256) / 256.0
    B = wl.DT_BF16
    rows = []

    def time_first(model, batch=1):
        h = ec.Model(pool, model, wl.to_storage(model.weights, model.dtype), max_batch=batch)
        h.alloc_set([sid] * model.n_groups)
        if tune:
            h.tune(sid, batch, 2)
        ns = h.profile_group(0, sid, batch, 5)[0]
        info = h.kernel_info(0, sid, batch)
        h.free()
        return ns, info

    def mem(name, model, nbytes, batch=1):
        ns, info = time_first(model, batch)
        rows.append((name, info["kernel"], "hbm", nbytes / ns, HBM_PEAK_GBS, "GB/s", ns / 1e3))

    def gemm(name, m_, k_, n_):
        bb = G._Builder(name, B, 0, G.IN_SEQ, k_, 1, m_)
        x = bb.linear(-1, n_, std=0.02)
        bb.eltwise(x)                       # keeps the GEMM's output in the 16-bit type
        ns, info = time_first(bb.finish())
        tf = 2.0 * m_ * k_ * n_ / ns / 1e3
        rows.append((f"{name} M{m_} N{n_} K{k_} tile {info['tile'][0]}x{info['tile'][1]}", info["kernel"], "mfma", tf,
                     mfma_peak, "TFLOP/s", ns / 1e3))

    # every case is a two-layer model whose first layer is the kernel under test (so that it writes the 16-bit type)
    def c_ln():
        bb = G._Builder("ln", B, 0, G.IN_SEQ, 1024, 1, 480000); x = bb.layernorm(-1); bb.softmax(x)
        mem("LayerNorm, 480000 rows x 1024", bb.finish(), 480000 * 1024 * 4)

    def c_sm():
        bb = G._Builder("sm", B, 0, G.IN_SEQ, 384, 1, 960000); x = bb.softmax(-1); bb.softmax(x)
        mem("softmax, 960000 rows x 384", bb.finish(), 960000 * 384 * 4)

    def c_mp():
        bb = G._Builder("mp", B, 0, G.IN_IMAGE, 64, 1792, 1792); x = bb.maxpool(-1, 3, 2, 1); bb.gap(x)
        mem("max-pool 3x3 s2, 64 x 1792 x 1792", bb.finish(), 64 * 1792 * 1792 * 2 + 64 * 896 * 896 * 2)

    def c_dw():
        bb = G._Builder("dw", B, 0, G.IN_IMAGE, 192, 1120, 1120); x = bb.conv(-1, 192, 3, 1, 1, G.ACT_RELU6, groups=192); bb.gap(x)
        mem("depthwise 3x3 + ReLU6, 192 x 1120 x 1120", bb.finish(), 192 * 1120 * 1120 * 4)

    def c_gap():
        bb = G._Builder("gap", B, 0, G.IN_IMAGE, 2048, 224, 224); x = bb.gap(-1); bb.softmax(x)
        mem("global average pool, 4 x 2048 x 224 x 224", bb.finish(), 4 * 2048 * 224 * 224 * 2, batch=4)

    def c_gelu():
        bb = G._Builder("el", B, 0, G.IN_SEQ, 1024, 1, 480000); x = bb.eltwise(-1, G.ACT_GELU, bias_std=1.0); bb.eltwise(x)
        mem("bias + GELU, 480000 x 1024", bb.finish(), 480000 * 1024 * 4)

    def c_copy():
        bb = G._Builder("cp", B, 0, G.IN_SEQ, 1024, 1, 480000); x = bb.eltwise(-1); bb.eltwise(x)
        mem("plain copy (element-wise, no bias, no activation), 480000 x 1024", bb.finish(), 480000 * 1024 * 4)

    def c_fc():
        bb = G._Builder("fc", B, 0, G.IN_SEQ, 25088, 1, 8); x = bb.linear(-1, 4096, std=0.01); bb.eltwise(x)
        ns, info = time_first(bb.finish())
        nbytes = 2 * (8 * 25088 + 4096 * 25088 + 8 * 4096)
        rows.append(("VGG FC1 b8: linear M8 N4096 K25088 (weight streaming)", info["kernel"], "hbm", nbytes / ns, HBM_PEAK_GBS, "GB/s", ns / 1e3))

    def c_attn(batch):
        # fused attention of BERT-large (16 heads of 64, 384 keys): 4 B S Hd elements move, 4 B S^2 Hd flops -- S / 2 = 192
        # flop per byte, below the ridge, so the row is held against the memory roofline
        bb = G._Builder("attn", B, 0, G.IN_SEQ, 3 * 1024, 1, 384); x = bb.attention(-1, 16); bb.eltwise(x)
        ns, info = time_first(bb.finish(), batch)
        nbytes = 2.0 * 4 * batch * 384 * 1024
        rows.append((f"attention 16 x 64, 384 keys, batch {batch} ({4.0 * batch * 384 * 384 * 1024 / ns / 1e3:.0f} TFLOP/s)", info["kernel"], "hbm",
                     nbytes / ns, HBM_PEAK_GBS, "GB/s", ns / 1e3))

    cases = [("attention", lambda: c_attn(256)), ("attention_b4", lambda: c_attn(4)), ("layernorm", c_ln), ("softmax", c_sm), ("maxpool", c_mp), ("dwconv", c_dw), ("gap", c_gap), ("gelu", c_gelu),
             ("copy", c_copy), ("fc", c_fc),
             ("gemm8192", lambda: gemm("linear", 8192, 8192, 8192)), ("gemm4096", lambda: gemm("linear", 4096, 4096, 4096)),
             ("ffn1", lambda: gemm("BERT-large FFN1 b4", 1536, 1024, 4096)), ("ffn2", lambda: gemm("BERT-large FFN2 b4", 1536, 4096, 1024)),
             ("qkv", lambda: gemm("BERT-large QKV b4", 1536, 1024, 3072)),
             ("proj", lambda: gemm("BERT-large projection b4", 1536, 1024, 1024)),
             ("base_ffn1", lambda: gemm("BERT-base FFN1 b1", 128, 768, 3072))]
    for key, fn in cases:
        if (only is None and not extra_gemms) or (only is not None and key in only.split(",")):
            fn()
    for shape in (extra_gemms or "").split(";"):
        if shape:
            m_, n_, k_ = (int(v) for v in shape.split(","))
            gemm("linear", m_, k_, n_)
    pool.destroy()
    if cus < 256:
        print(f"# on a stream masked to {cus} CUs; matrix-core rows against {mfma_peak:.1f} TFLOP/s = 2500 x {cus} / 256")
    print(f"{'case':66s} {'kernel':18s} {'bound':5s} {'achieved':>10s} {'peak':>8s} {'unit':8s} {'frac':>6s} {'us/launch':>10s}")
    for name, kern, bound, ach, peak, unit, us in rows:
        print(f"{name:66s} {kern:18s} {bound:5s} {ach:10.1f} {peak:8.0f} {unit:8s} {ach / peak:6.3f} {us:10.1f}")


# ---------------------------------------------------------------------------------------------------
# hardware characterisation (the paper's Sec. II-C experiments, on this GPU)
# ---------------------------------------------------------------------------------------------------
def characterize_mode():
    import collections
    import paper_2506_12598_amd as ec

    def words(bits):
        return ec.words_of_bits(bits, 8)

    print("== CU-mask geometry (eclip_pool_probe: hardware ids of 4096 one-wave workgroups per mask)")
    cases = [("unmasked", None), ("bits 0-31", words(range(32))), ("bits 0-7", words(range(8))),
             ("bits i with i%16<8", words([i for i in range(256) if i % 16 < 8])), ("bits 128-255", words(range(128, 256))),
             ("layout worker 0, 2 granules of 32", ec.eclip_mask_layout(256, 32, 2, 0, 2)),
             ("layout worker 1, 2 granules of 32", ec.eclip_mask_layout(256, 32, 2, 1, 2)),
             ("layout worker 0, 1 granule of 64, stripe 8", ec.eclip_mask_layout(256, 64, 2, 0, 1, 8))]
    pool = ec.Pool([(w, -1) for _, w in cases])
    for i, (name, _) in enumerate(cases):
        ids = pool.probe(i, 4096).tolist()
        cus = set(ids)
        per_xcd = collections.Counter(v >> 16 for v in cus)
        ses = sorted({(v >> 8) & 0xff for v in cus})
        wg_xcd = collections.Counter(v >> 16 for v in ids)
        print(f"  {name:44s} distinct CUs {len(cus):3d}; CUs per XCD {sorted(per_xcd.values())}; shader engines used {ses}; "
              f"workgroups per XCD {min(wg_xcd.values())}..{max(wg_xcd.values())}")
    print("  (a mask that leaves an XCD without a CU is refused by eclip_pool_create: the runtime crashes on it)")
    pool.destroy()

    print("== repartitioning cost (Observation 1): wall time per kernel of a dependent chain of trivial kernels")
    pool = ec.Pool([(words(range(32 * g, 32 * g + 32)), -1) for g in range(4)])
    same, pooled, create = pool.bench_switch(0, 1, 3000)
    print(f"  same stream {same / 1e3:8.2f} us | alternating two pooled masked streams {pooled / 1e3:8.2f} us | "
          f"a new masked stream per kernel {create / 1e3:10.2f} us")
    pool.destroy()

    print("== number of masked streams vs latency (Observation 2): chain dealt round-robin over n streams of 8 CUs")
    pool = ec.Pool([(words(range(8 * g, 8 * g + 8)), -1) for g in range(12)])
    for n in range(1, 13):
        t = pool.bench_streams(list(range(n)), 1500)
        print(f"  n = {n:2d}: {t / 1e3:9.2f} us per kernel")
    print("== pairs of streams: chain alternating between streams i and j (creation ranks), us per kernel")
    print("       " + " ".join(f"j={j:<5d}" for j in range(1, 9)))
    for i in range(0, 8):
        row = []
        for j in range(1, 9):
            row.append(f"{pool.bench_streams([i, j], 600) / 1e3:7.1f}" if j > i else "      .")
        print(f"  i={i}  " + " ".join(row))
    pool.destroy()


# ---------------------------------------------------------------------------------------------------
# the paper's partitioning scenarios side by side (Sec. IV "Spatial Partitioning Scenarios", Table I) and the
# per-kernel optimizer with a sweep of the switch budget (Sec. III-B)
# ---------------------------------------------------------------------------------------------------
def policies_mode(args):
    import dataclasses
    import torch
    import workloads as wl
    import paper_2506_12598_amd as ec

    cfg = args.config
    steps = args.steps if args.steps is not None else {1: 1000, 2: 500, 3: 200, 4: 20, 6: 300, 7: 300}[cfg]
    warmup = args.warmup if args.warmup is not None else {1: 100, 2: 50, 3: 20, 4: 2, 6: 30, 7: 30}[cfg]
    configs = [32, 64, 128, 192, 256]
    full = len(configs) - 1
    stage_models = wl.config_models(cfg if cfg <= 4 else cfg - 1)
    n_w = len(stage_models)
    # one kernel group per kernel: the unit of the paper's model
    models = [dataclasses.replace(m, group_of_layer=list(range(len(m.layers))), n_groups=len(m.layers)) for m in stage_models]
    batches = [[4]] * 3 + [[8]] if cfg == 4 else [[1]] * n_w
    pb = [b[0] for b in batches]

    masks, prof_id = [], {}
    for w in range(n_w):
        for ci, c in enumerate(configs):
            prof_id[(w, ci)] = len(masks)
            masks.append((ec.eclip_mask_layout(256, 32, n_w, w, c // 32), w))
    prof_pool = ec.Pool(masks)
    workers = [Worker(ec, torch, prof_pool, m, i, args.depth, batches[i]) for i, m in enumerate(models)]
    # beta[w][k][c]: latency of kernel k of worker w on configuration c, in ns (Sec. III-B, factor (i))
    beta = [[[int(wk.h.profile_group(k, prof_id[(w, ci)], batch=pb[w], iters=3 if cfg == 4 else 40)[0]) for ci in range(len(configs))]
             for k in range(len(wk.model.layers))] for w, wk in enumerate(workers)]
    switch_cost_ns = measured_switch_cost_ns(prof_pool, prof_id[(0, 0)], prof_id[(0, 1)])
    log(f"config {cfg}: {[len(m.layers) for m in models]} kernels per worker profiled on {configs} CUs; switch cost {switch_cost_ns} ns")

    def predicted_us(assign):
        """The model's objective for an assignment: sum over workers of solo latency x (1 + alpha), alpha from the
        CUs by which the workers' kernel-weighted average allocations exceed the GPU (Sec. III-B), in us."""
        tot_b, s_avg = 0.0, 0.0
        for w, a in enumerate(assign):
            tot_b += sum(beta[w][k][c] for k, c in enumerate(a))
            s_avg += sum(configs[c] for c in a) / len(a)
        return tot_b * (1.0 + max(0.0, s_avg - 256.0) / 256.0) / 1e3

    ones = [[1] * len(m.layers) for m in models]
    policies = []                                       # (name, per-kernel configuration index per worker or None = unmasked)
    policies.append(("Baseline: one shared unmasked stream", "shared"))
    policies.append(("Unpartitioned: one unmasked stream per worker", None))
    # Model-Wise (Sec. II-A, Sec. IV): the fewest CUs whose whole-model latency stays within slo x the latency on all CUs
    mw, _ = ec.eclip_alloc_model_wise(configs, beta, int(round(args.slo * 100)), 100)
    policies.append((f"Model-Wise (fewest CUs within {args.slo:g}x solo latency)", mw))
    # Kernel-Wise on pooled streams (Sec. IV): every kernel at its minimum-CU threshold (within 5 % of its latency on all CUs)
    kw, _ = ec.eclip_alloc_kernel_wise(configs, beta, 5)
    policies.append(("KW-Prealloc (every kernel at its own CU knee, pooled streams)", kw))
    # ECLIP on the stage groups bench.py uses by default
    g_beta = [[[sum(beta[w][k][ci] for k in range(len(m.layers)) if m.group_of_layer[k] == g) for ci in range(len(configs))]
               for g in range(m.n_groups)] for w, m in enumerate(stage_models)]
    g_nk = [[sum(1 for k in m.group_of_layer if k == g) for g in range(m.n_groups)] for m in stage_models]
    mc = max(1, 4 // n_w)
    a_g, _, _ = ec.eclip_alloc_solve(256, configs, g_nk, g_beta, args.switch_max, max_configs=mc, switch_cost_ns=switch_cost_ns)
    policies.append((f"ECLIP, stage groups, switchMax {args.switch_max}, <= {mc} configs/worker, switch cost",
                     [[a_g[w][m.group_of_layer[k]] for k in range(len(m.layers))] for w, m in enumerate(stage_models)]))
    # ECLIP on single kernels: the optimizer derives the groups; sweep of the switch budget.  (The exact solver's state
    # space grows with units x switch budget x CU sums; workers of 150+ kernels exceed its budget, and the sweep is
    # then limited to what it accepts.)
    def per_kernel(label, sm, **kw):
        try:
            a, _, _ = ec.eclip_alloc_solve(256, configs, ones, beta, sm, **kw)
            policies.append((label, a))
        except ec.EclipError as err:
            if err.status != ec.ELIMIT:
                raise
            log(f"{label}: not solved ({err})")
    per_kernel(f"ECLIP, per kernel, switchMax {args.switch_max}, <= {mc} configs/worker, switch cost", args.switch_max,
               max_configs=mc, switch_cost_ns=switch_cost_ns)
    # the budget alone (no price on a switch), as in the paper: how much do the switches it allows cost here?
    for sm in (0, 2, 4, 8, 14, 28):
        per_kernel(f"ECLIP, per kernel, switchMax {sm}, <= {mc} configs/worker, no switch cost", sm, max_configs=mc)
    per_kernel(f"ECLIP, per kernel, switchMax {args.switch_max}, model as printed (no stream limit, no switch cost)", args.switch_max)

    rows = []
    pool = prof_pool
    for name, assign in policies:
        masks = [(None, -1)] + [(None, w) for w in range(n_w)]
        mask_id = {}
        if assign not in (None, "shared"):
            for w in range(n_w):
                for c in sorted(set(assign[w])):
                    mask_id[(w, c)] = len(masks)
                    masks.append((ec.eclip_mask_layout(256, 32, n_w, w, configs[c] // 32), w))
        new_pool = ec.Pool(masks)
        for wk in workers:
            wk.h.rebind(new_pool)
        pool.destroy()
        pool = new_pool
        for w, wk in enumerate(workers):
            if assign == "shared": wk.h.alloc_set([0] * len(wk.model.layers))
            elif assign is None: wk.h.alloc_set([1 + w] * len(wk.model.layers))
            else: wk.h.alloc_set([mask_id[(w, c)] for c in assign[w]])
        sw = [wk.h.switches() for wk in workers]
        run_closed(workers, warmup)
        torch.cuda.synchronize()
        dt, served = run_closed(workers, steps)
        torch.cuda.synchronize()
        cus = "-" if assign in (None, "shared") else " | ".join(
            ",".join(f"{configs[c]}x{n}" for c, n in _runs(a)) for a in assign)
        rows.append({"policy": name, "inferences_per_s": served / dt, "ms_per_step": 1e3 * dt / steps, "switches_per_request": sw,
                     "streams_in_use": len(masks) - 1 - n_w if assign not in (None, "shared") else 1 if assign == "shared" else n_w,
                     "predicted_us": None if assign in (None, "shared") else predicted_us(assign), "allocation": cus})
        log(f"{name}: {rows[-1]['inferences_per_s']:.0f} inf/s, switches {sw}")
    for wk in workers:
        wk.h.free()
    pool.destroy()
    note = " (every request at batch 1 in this mode)" if cfg == 3 else ""
    print(f"# {WORKLOADS[cfg]}{note}; closed loop, {args.depth} requests in flight per worker, {steps} steps; CU configurations {configs}")
    print("# every kernel is a kernel group of its own in this mode (the unit of the paper's model), so kernels of different layers "
          "never share a launch: absolute rates are below those of the default bench, which serves the stage groups")
    print(f"{'policy':98s} {'inf/s':>9s} {'ms/step':>8s} {'switches/request':>18s} {'streams':>7s} {'model us':>9s}")
    for r in rows:
        pu = "-" if r["predicted_us"] is None else f"{r['predicted_us']:.1f}"
        print(f"{r['policy']:98s} {r['inferences_per_s']:9.0f} {r['ms_per_step']:8.3f} {str(r['switches_per_request']):>18s} "
              f"{r['streams_in_use']:7d} {pu:>9s}")
    print("# allocations (CUs x consecutive kernels, per worker):")
    for r in rows:
        if r["allocation"] != "-":
            print(f"#   {r['policy'][:60]:60s} {r['allocation']}")


def _runs(a):
    out = []
    for c in a:
        if out and out[-1][0] == c: out[-1][1] += 1
        else: out.append([c, 1])
    return out


# ---------------------------------------------------------------------------------------------------
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 6, 7, 8],
                    help="co-location mix (4 = headline workload, the stress mix; 6, 7 = mixes of the second workload family)")
    ap.add_argument("--depth", type=int, default=2, help="requests each worker keeps in flight")
    ap.add_argument("--window", type=float, default=10.0, help="seconds of open-loop Poisson load per policy (0 = skip)")
    ap.add_argument("--graphs", type=int, default=0, choices=[0, 1], help="serve captured requests (HIP graphs replayed per stream segment)")
    ap.add_argument("--objective", default="energy", choices=["energy", "throughput"],
                    help="what picks the served allocation among the candidates: inferences per joule within the throughput floor, or throughput")
    ap.add_argument("--serve", default=None, metavar="NAME",
                    help="serve the candidate allocation whose name contains NAME in the timed region, whatever its trial says")
    ap.add_argument("--throughput-floor", type=float, default=0.85, help="with --objective energy: candidates below this fraction of the fastest trial are out")
    ap.add_argument("--trial-seconds", type=float, default=2.0)
    ap.add_argument("--energy-window", type=float, default=3.0, help="seconds of closed loop per policy and repeat for inferences/J (0 = skip)")
    ap.add_argument("--energy-repeats", type=int, default=3)
    ap.add_argument("--rate", type=float, default=None, help="Poisson arrivals/s per model (default: 200 for config 1, "
                                                             "else 70%% of the measured closed-loop rate)")
    ap.add_argument("--switch-max", type=int, default=14)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true", help="run only the per-layer timing pass behind the `roofline` entry and print it")
    ap.add_argument("--no-tune", action="store_true", help="keep the planner's cost-model choices (skip eclip_model_tune)")
    ap.add_argument("--policy", default="eclip", choices=["eclip", "unpart_a", "unpart_b"], help="policy of the timed region")
    ap.add_argument("--kernels", action="store_true", help="time single kernels at roofline shapes and print a table")
    ap.add_argument("--cus", type=int, default=256, help="with --kernels: run on a stream masked to this many CUs (a multiple of 16)")
    ap.add_argument("--gemm", default=None, help="with --kernels: time linear layers of these shapes, 'M,N,K;M,N,K;...'")
    ap.add_argument("--only", default=None, help="with --kernels: comma-separated case keys (layernorm, softmax, maxpool, dwconv, "
                    "gap, gelu, copy, fc, gemm8192, gemm4096, ffn1, ffn2, qkv, proj, base_ffn1)")
    ap.add_argument("--policies", action="store_true", help="compare the paper's partitioning scenarios and sweep the switch budget")
    ap.add_argument("--slo", type=float, default=3.0, help="with --policies: Model-Wise latency target as a multiple of solo latency")
    ap.add_argument("--pmc-copy", action="store_true", help="also run the calibration copy (for rocprofv3 --pmc runs)")
    ap.add_argument("--stats-from", default=None, metavar="KERNEL_TRACE_CSV",
                    help="reduce the kernel_trace CSV of a `rocprofv3 --kernel-trace` run of this file to per-kernel tables and exit")
    ap.add_argument("--counters-from", nargs="+", default=None, metavar="COUNTER_CSV",
                    help="reduce counter_collection CSVs of `rocprofv3 --pmc` runs of this file to per-kernel means and exit")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"), default=None,
                    help="reduce two rocprofv3 --pmc counter_collection CSVs to profiles/traffic_config<N>.json and exit")
    ap.add_argument("--characterize", action="store_true", help="CU-mask geometry, switch cost and stream-count sweep")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; co-located models are independent workers and would be "
              "placed on different GPUs without any exchange step. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.stats_from:
        stats_from(args.stats_from)
        return
    if args.counters_from:
        counters_from(args.counters_from)
        return
    if args.traffic_from:
        traffic_from(args.config, args.traffic_from[0], args.traffic_from[1],
                     "rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) --output-format csv -- python3 bench.py --pmc-copy "
                     f"--config {args.config} --roofline-only")
        return
    import torch
    import workloads as wl
    import paper_2506_12598_amd as ec
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.init()
    if args.kernels:
        kernels_mode(args.only, args.gemm, tune=not args.no_tune, cus=args.cus)
        return
    if args.characterize:
        characterize_mode()
        return
    if args.policies:
        policies_mode(args)
        return
    if args.pmc_copy:
        pmc_copy(ec, torch)
    time.sleep(0.5)
    idle_w = PowerSampler().read()          # board power before any kernel of this process has run

    cfg = args.config
    steps = args.steps if args.steps is not None else {1: 2000, 2: 1000, 3: 300, 4: 30, 6: 500, 7: 500, 8: 100}[cfg]
    warmup = args.warmup if args.warmup is not None else {1: 200, 2: 100, 3: 30, 4: 3, 6: 50, 7: 50, 8: 10}[cfg]
    # lengths of the untimed legs (calibration of the interference slope, trials between candidate allocations,
    # profiling samples): fixed per mix, whatever --steps says, so that a short timed region does not make them noisy
    n_cal = {1: 300, 2: 200, 3: 80, 4: 20, 6: 100, 7: 100, 8: 40}[cfg]
    prof_iters = 40 if cfg != 4 else 20
    # CU configurations: the stress mix sweeps 16..256 in steps of 16 (2 CUs per XCD and granule, so no XCD is ever
    # left empty); the other mixes use the five-entry pool of their configuration
    granule = 16 if cfg == 4 else 32
    configs = [32, 64, 128, 192, 256] if cfg != 4 else list(range(16, 257, 16))
    models = wl.config_models(cfg if cfg <= 4 else cfg - 1)
    n_w = len(models)
    if cfg == 3:
        rng = np.random.default_rng(77)
        batches = [[int(b) for b in rng.integers(1, 9, size=64)] for _ in models]
    elif cfg == 4:
        batches = [[4]] * 3 + [[8]]
    elif cfg == 8:
        batches = [[8], [4]]
    else:
        batches = [[1]] * n_w
    prof_batch = [max(1, int(round(np.mean(b)))) for b in batches]

    # ---- profiling pool: every configuration of every worker, laid out per worker as in Sec. III-A
    masks = []
    prof_id = {}
    for w in range(n_w):
        for ci, c in enumerate(configs):
            prof_id[(w, ci)] = len(masks)
            masks.append((ec.eclip_mask_layout(256, granule, n_w, w, c // granule), w))
    t0 = time.perf_counter()
    prof_pool = ec.Pool(masks)
    workers = [Worker(ec, torch, prof_pool, m, i, args.depth, batches[i]) for i, m in enumerate(models)]
    log(f"config {cfg}: loaded {n_w} models in {time.perf_counter() - t0:.1f}s, profiling pool of {len(masks)} masked streams")

    def measure_roofline(pool):
        # ---- roofline of the dominant kernel: HIP-event timings on the stream the kernels run on.  Each layer of each
        # model is timed on that worker's unpartitioned stream (8 back-to-back launches per sample, see
        # eclip_profile_group); layers are grouped by the kernel function that runs them; the matrix-core function
        # with the largest launch-weighted time is reported against the roofline that bounds its work.
        for w, wk in enumerate(workers):
            wk.h.alloc_set([1 + w] * wk.model.n_groups)
        pool.probe(0, 8)                 # marks the start of this pass in a kernel trace (see --stats-from)
        per_kernel = {}
        for w, wk in enumerate(workers):
            ns_all = []
            for g in range(wk.model.n_groups):
                ns_all.extend(wk.h.profile_group(g, 1 + w, batch=prof_batch[w], iters=20 if cfg != 4 else 10))
            work = gemm_work(wk.model, prof_batch[w])
            for li, ns in enumerate(ns_all):
                info = wk.h.kernel_info(li, 1 + w, prof_batch[w])
                e = per_kernel.setdefault(info["kernel"], {"ns": 0.0, "bytes": 0.0, "flops": 0.0, "launches": 0, "layers": 0})
                e["ns"] += ns
                e["launches"] += info["launches"]
                e["layers"] += 1
                if work[li] is not None:
                    e["bytes"] += work[li][0]
                    e["flops"] += work[li][1]
        pool.probe(0, 8)                 # ... and its end
        total_ns = sum(v["ns"] for v in per_kernel.values())
        # a layer whose K is cut over the grid runs two kernels (GEMM + slice sum): its time is attributed per launch
        dom = max((k for k in per_kernel if per_kernel[k]["bytes"] > 0),
                  key=lambda k: per_kernel[k]["ns"] * per_kernel[k]["layers"] / per_kernel[k]["launches"])
        d = per_kernel[dom]
        ai = d["flops"] / d["bytes"]
        if ai > RIDGE:
            ach, peak, unit, bound = d["flops"] / d["ns"] / 1e3, MFMA_PEAK_TFLOPS, "TFLOP/s", "mfma"
        else:
            ach, peak, unit, bound = d["bytes"] / d["ns"], HBM_PEAK_GBS, "GB/s", "hbm"
        # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counters of an earlier profiled run of this workload;
        # null when there is none or when a kernel source has changed since
        traffic = None
        if os.path.exists(traffic_path(cfg)):
            t = json.load(open(traffic_path(cfg)))
            if t.get("source_sha256") == source_hash() and dom in t["kernels"]:
                traffic = t["kernels"][dom]["fetch_bytes_per_launch"] + t["kernels"][dom]["write_bytes_per_launch"]
        roofline = {"bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak, "traffic": traffic,
                    "kernel": dom, "flop_per_byte": ai, "layers_per_step": d["layers"], "launches_per_step": d["launches"],
                    "avg_layer_us": d["ns"] / d["layers"] / 1e3, "avg_bytes_per_layer": d["bytes"] / d["layers"],
                    "achieved_tflops": d["flops"] / d["ns"] / 1e3, "achieved_gbs": d["bytes"] / d["ns"],
                    "time_share_by_kernel": {k: v["ns"] / total_ns for k, v in per_kernel.items()}}
        return roofline

    if args.roofline_only:
        # only the per-layer timing pass behind the `roofline` entry: models on one full-GPU stream each (the unpartitioned
        # policy), plans tuned for that CU count.  Short enough to run under a profiler with a trace small enough to keep.
        all_cus = ec.eclip_mask_layout(256, 256, 1, 0, 1)
        pool = ec.Pool([(None, -1)] + [(all_cus, w) for w in range(n_w)])
        for wk in workers:
            wk.h.rebind(pool)
        prof_pool.destroy()
        if not args.no_tune:
            for w, wk in enumerate(workers):
                for b in sorted(set(wk.batches)):
                    wk.h.tune(1 + w, batch=b, iters=1)
        print(json.dumps({"roofline": measure_roofline(pool), "n_gpus": 1, "data": "synthetic",
                          "config": {"workload": WORKLOADS[cfg], "leg": "per-layer timing pass only"}}))
        torch.cuda.synchronize()
        for wk in workers:
            wk.h.free()
        pool.destroy()
        return

    # ---- latency-vs-CU tables (Sec. III-B profiling), the measured cost of a switch, and the allocation.
    # Every group is timed as eclip_submit serves it (launch sharing and input re-layout included); the kernel count
    # that weighs a group in CUAverage is the number of launches it makes.
    t0 = time.perf_counter()
    # measured plan selection first (eclip_model_tune): which tile shape serves every GEMM problem best on every CU count
    if not args.no_tune:
        n_tuned = 0
        for w, wk in enumerate(workers):
            for ci in range(len(configs)):
                for b in sorted(set(wk.batches)):
                    n_tuned += wk.h.tune(prof_id[(w, ci)], batch=b, iters=1)
        log(f"tuned {n_tuned} (GEMM problem, CU count) pairs in {time.perf_counter() - t0:.1f}s")
    beta, nk = [], []
    for w, wk in enumerate(workers):
        rows, counts = [], []
        for g in range(wk.model.n_groups):
            prof = [wk.h.profile_group_served(g, prof_id[(w, ci)], batch=prof_batch[w], iters=prof_iters) for ci in range(len(configs))]
            rows.append([int(ns) for ns, _ in prof])
            counts.append(max(1, prof[-1][1]))
        beta.append(rows); nk.append(counts)
    switch_cost_ns = measured_switch_cost_ns(prof_pool, prof_id[(0, 0)], prof_id[(0, 1)])
    # The GPU serves one queue per compute pipe at a time (4 pipes), so at most 4 masked streams may be in use over
    # all workers.  The solver's limit is per worker, so the global budget is spent by enumeration: one solve per way
    # of dealing 4 streams to the workers (at least one each), best objective kept (solve_within_streams).
    max_configs = max(1, 4 // n_w)

    def compositions(total, parts):
        if parts == 1:
            return [(total,)]
        return [(k,) + rest for k in range(1, total - parts + 2) for rest in compositions(total - k, parts - 1)]

    def solve_within_streams(per_worker_cap, sc, kw):
        """Best allocation with at most 4 streams in use overall and at most `per_worker_cap` per worker."""
        best = None
        for comp in compositions(max(4, n_w), n_w):
            comp = [min(k, per_worker_cap) for k in comp]
            a, obj, sw = ec.eclip_alloc_solve(256, configs, nk, beta, args.switch_max, switch_cost_ns=sc, max_configs_of_worker=comp, **kw)
            if best is None or obj < best[1]:
                best = (a, obj, sw)
        return best
    # Slope of the interference law.  The model charges a kernel (1 + alpha) times its solo latency, alpha = CU overlap /
    # total CUs, a slope the paper calibrated on its GPU (two kernels on the same CUs: twice as long).  Here the slope is
    # measured with the mix itself: every worker alone, then all together, each time on its full-GPU mask (overlap =
    # (n_w - 1) x all CUs).  The solver takes the calibrated law as an alpha table over the overlap, in granule steps.
    full = len(configs) - 1
    for w, wk in enumerate(workers):
        wk.h.alloc_set([prof_id[(w, full)]] * wk.model.n_groups)
    solo_rate = []
    for wk in workers:
        dt, served = run_closed_for([wk], n_cal, seconds=0.5)
        solo_rate.append(served / dt)
    dt, _ = run_closed_for(workers, n_cal)
    co_rate = [wk.served / dt for wk in workers]
    torch.cuda.synchronize()
    slowdown = float(np.mean([s / max(c, 1e-9) for s, c in zip(solo_rate, co_rate)]))
    slope = min(1.0, max(0.02, (slowdown - 1.0) / max(1, n_w - 1)))
    alpha_ppm = [int(round(slope * (k * granule / 256.0) * 1e6)) for k in range((n_w - 1) * (256 // granule) + 1)]
    # Candidate allocations.  First the model exactly as printed in Sec. III-B (slope 1, the switch budget as the only
    # limit on switches) -- always served and reported, whatever it costs here.  Then the model with this GPU's two
    # limits added (at most 4 streams in use, a price per switch), with the paper's slope and with the measured one,
    # each also restricted to one configuration per worker (no switches).  When they differ, each serves a short
    # closed-loop trial on its own serving pool and the fastest is kept: the (1 + alpha) law is coarse on this GPU either
    # way (small kernels hardly interfere, a switch costs more inside a pipelined request stream than in isolation), so
    # the profile picks the candidates and a measurement picks between them.
    cand = []
    table = {"overlap_mode": ec.OVERLAP_TABLE, "alpha_ppm": alpha_ppm, "granule": granule}
    for name, kw, mc, sc in (("model as printed (Sec. III-B: slope 1, switch budget only)", {}, 0, 0),
                             ("paper slope", {}, 4, switch_cost_ns), ("measured slope", table, 4, switch_cost_ns),
                             ("paper slope, one configuration per worker", {}, 1, switch_cost_ns),
                             ("measured slope, one configuration per worker", table, 1, switch_cost_ns)):
        if mc == 0:
            a, _, sw = ec.eclip_alloc_solve(256, configs, nk, beta, args.switch_max, switch_cost_ns=sc, **kw)
        else:
            a, _, sw = solve_within_streams(mc, sc, kw)
        if not any(a == c[1] for c in cand):
            cand.append((name, a, sw))
    # ... and the corner of the configuration space where nothing is partitioned: every worker on a mask of all CUs.  The
    # (1 + alpha) law misjudges that corner by 10-15 % on this GPU in either direction (workgroups of different kernels
    # interleave on a compute unit more gracefully than "twice as long"), so it is always part of the trial.
    # ... the plain static partition: equal disjoint shares, 256 / workers CUs each (what Model-Wise gives identical workers)
    if 256 // n_w in configs and n_w > 1:
        a_eq = [[configs.index(256 // n_w)] * m.n_groups for m in models]
        if not any(a_eq == c[1] for c in cand):
            cand.append(("equal disjoint shares", a_eq, [0] * n_w))
    a_full = [[full] * m.n_groups for m in models]
    if not any(a_full == c[1] for c in cand):
        cand.append(("every worker on all CUs (masked streams, full overlap)", a_full, [0] * n_w))
    log(f"profiled in {time.perf_counter() - t0:.1f}s; switch cost {switch_cost_ns} ns; co-run slowdown {slowdown:.3f} -> "
        f"overlap slope {slope:.3f}; candidates " + "; ".join(f"{n}: {[_runs([configs[c] for c in w]) for w in a]}" for n, a, _ in cand))

    # ---- serving pool: id 0 = shared unmasked stream (policy unpart_a); ids 1..n_w = one private unmasked stream per
    # worker (policy unpart_b); then only the masked streams the allocation uses, created back to back so that they
    # land on distinct pipes
    # (the private streams of policy unpart_b carry a mask of all CUs rather than no mask: a masked stream owns a hardware
    # queue, while plain streams are dealt onto the runtime's few shared queues, where two workers can land on the same one
    # and serialise -- measured on the stress mix: 2780 against 3420 inf/s from one run to the next with plain streams)
    all_cus = ec.eclip_mask_layout(256, 256, 1, 0, 1)

    def serving_pool(assign):
        masks = [(None, -1)] + [(all_cus, w) for w in range(n_w)]
        mask_id = {}
        for w in range(n_w):
            for c in sorted(set(assign[w])):
                mask_id[(w, c)] = len(masks)
                masks.append((ec.eclip_mask_layout(256, granule, n_w, w, configs[c] // granule), w))
        pool = ec.Pool(masks)
        return pool, [[mask_id[(w, c)] for c in assign[w]] for w in range(n_w)]

    # Every candidate serves a trial on a serving pool of its own: closed loop, warm-up, then `--trial-seconds` with the
    # board power sampled.  The profiling pool goes before the trials and a candidate's pool goes right after its trial:
    # dozens of idle queues next to the serving streams slow dispatch down several times over (measured: the same
    # allocation 816 inf/s with the 64-stream pool alive, 3100 without).
    # Selection (`--objective`): "energy" (default) takes the candidate with the most inferences per joule among those
    # within `--throughput-floor` (0.85) of the fastest trial; "throughput" takes the fastest.
    for wk in workers:
        wk.h.graphs(bool(args.graphs))
    trials = []
    sampler = PowerSampler()
    prev_pool = prof_pool
    for name, a, sw in cand:
        pool_c, table_c = serving_pool(a)
        for wk, t in zip(workers, table_c):
            wk.h.rebind(pool_c)
            wk.h.alloc_set(t)
        prev_pool.destroy()
        prev_pool = pool_c
        run_closed_for(workers, n_cal, seconds=0.3)
        sampler.start()
        time.sleep(0.05)
        t_a = time.perf_counter()
        dt, served = run_closed_for(workers, n_cal, seconds=args.trial_seconds, warm_seconds=0.0)
        torch.cuda.synchronize()
        t_b = time.perf_counter()
        sampler.stop()
        e = sampler.energy_j(t_a, t_b)
        rate = served / dt
        ipj = None if not e else rate * (t_b - t_a) / e          # the window holds a short lead-in at the same load
        log(f"trial, {name}: {rate:.0f} inf/s, {ipj if ipj is None else round(ipj, 4)} inf/J")
        trials.append((rate, name, a, sw, ipj))
    fastest = max(t[0] for t in trials)
    if args.objective == "throughput" or any(t[4] is None for t in trials):
        best_i = max(range(len(trials)), key=lambda i: trials[i][0])
    else:
        ok = [i for i in range(len(trials)) if trials[i][0] >= args.throughput_floor * fastest]
        best_i = max(ok, key=lambda i: trials[i][4])
    if args.serve:
        # serve a named candidate whatever its trial says (e.g. "as printed": the pure Sec. III-B output, switches and all)
        hits = [i for i, t in enumerate(trials) if args.serve.lower() in t[1].lower()]
        if not hits:
            raise SystemExit(f"--serve {args.serve!r} matches none of: {[t[1] for t in trials]}")
        best_i = hits[0]
    _, chosen, assign, switches, _ = trials[best_i]
    pool, eclip_table = serving_pool(assign)
    for wk in workers:
        wk.h.rebind(pool)
    prev_pool.destroy()
    log(f"allocation ({chosen}) (CUs) {[[configs[c] for c in a] for a in assign]} switches {switches}")
    tables = {
        "eclip": eclip_table,
        "unpart_a": [[0] * m.n_groups for m in models],
        "unpart_b": [[1 + w] * m.n_groups for w, m in enumerate(models)],
    }

    def set_policy(name):
        for wk, t in zip(workers, tables[name]):
            wk.h.alloc_set(t)

    # ---- closed-loop throughput: the timed region is the last policy run
    closed = {}
    order = [p for p in ("unpart_a", "unpart_b", "eclip") if p != args.policy] + [args.policy]
    for pol in order:
        set_policy(pol)
        run_closed(workers, warmup)
        torch.cuda.synchronize()
        dt, served = run_closed(workers, steps)
        torch.cuda.synchronize()
        closed[pol] = {"inferences_per_s": served / dt, "ms_per_step": 1e3 * dt / steps}
        log(f"closed loop {pol}: {closed[pol]['inferences_per_s']:.0f} inf/s, {closed[pol]['ms_per_step']:.3f} ms/step")
    value = closed[args.policy]["inferences_per_s"]
    ms_per_step = closed[args.policy]["ms_per_step"]

    # ---- parity in this launch configuration: the last request of EVERY worker of the timed run
    last_out = []
    for wk in workers:
        b = wk.batches[(steps - 1) % len(wk.batches)]
        last_out.append((b, wk.d_out[(steps - 1) % args.depth][:b].cpu().numpy().astype(np.float64)))

    # ---- closed-loop energy: the same closed loop kept up for `--energy-window` seconds per policy, `--energy-repeats`
    # times, board power sampled at 20 Hz; inferences per joule with the spread over the repeats
    if args.energy_window > 0:
        sampler = PowerSampler()
        n_e = max(steps, int(args.energy_window * 1e3 / max(ms_per_step, 1e-3)))
        for pol in ("unpart_a", "unpart_b", "eclip"):
            set_policy(pol)
            n_pol = max(1, int(n_e * ms_per_step / closed[pol]["ms_per_step"]))
            vals, watts, mhz = [], [], []
            for _ in range(args.energy_repeats):
                sampler.start()
                time.sleep(0.1)
                t_a = time.perf_counter()
                dt, served = run_closed(workers, n_pol)
                torch.cuda.synchronize()
                t_b = time.perf_counter()
                sampler.stop()
                e = sampler.energy_j(t_a, t_b)
                if e:
                    vals.append(served / e)
                    watts.append(e / (t_b - t_a))
                    c = sampler.mean_clock_mhz(t_a, t_b)
                    if c:
                        mhz.append(c)
            if vals:
                closed[pol].update({"inferences_per_joule": float(np.mean(vals)), "inferences_per_joule_min": float(min(vals)),
                                    "inferences_per_joule_max": float(max(vals)), "avg_power_w": float(np.mean(watts)),
                                    "energy_windows": len(vals), "energy_window_s": float(n_pol * closed[pol]["ms_per_step"] / 1e3),
                                    "avg_sclk_mhz": float(np.mean(mhz)) if mhz else None})
                log(f"closed loop {pol}: {np.mean(vals):.4f} inf/J (min {min(vals):.4f}, max {max(vals):.4f}) at {np.mean(watts):.0f} W"
                    + (f", shader clock {np.mean(mhz):.0f} MHz" if mhz else ""))

    # ---- open loop: Poisson arrivals, p99 latency, energy
    open_res = {}
    if args.window > 0:
        sampler = PowerSampler()
        rate = args.rate if args.rate is not None else (200.0 if cfg == 1 else 0.7 * 1e3 / ms_per_step)
        for pol in ("unpart_a", "unpart_b", "eclip"):
            set_policy(pol)
            arr = [wl.poisson_arrivals(rate, args.window, i) for i in range(n_w)]
            lats = [[] for _ in workers]
            sampler.start()
            t_start = time.perf_counter() + 0.05
            th = [threading.Thread(target=wk.open_loop, args=(arr[i], t_start, lats[i])) for i, wk in enumerate(workers)]
            [t.start() for t in th]
            [t.join() for t in th]
            t_end = time.perf_counter()
            sampler.stop()
            allv = np.concatenate([np.array(l) for l in lats])
            served = sum(wk.served for wk in workers)
            e = sampler.energy_j(t_start, t_end)
            open_res[pol] = {
                "offered_requests_per_s": rate * n_w,
                "completed_requests": int(allv.size),
                "inferences_per_s": float(served / (t_end - t_start)),
                "p50_latency_ms": float(np.percentile(allv, 50) * 1e3),
                "p99_latency_ms": float(np.percentile(allv, 99) * 1e3),
                "p99_latency_ms_per_model": [float(np.percentile(np.array(l), 99) * 1e3) for l in lats],
                "avg_power_w": None if e is None else e / (t_end - t_start),
                "inferences_per_joule": None if e is None else float(served / e),
            }
            log(f"open loop {pol}: p99 {open_res[pol]['p99_latency_ms']:.3f} ms, {open_res[pol]['inferences_per_joule']} inf/J")
        open_res["idle_power_w"] = idle_w
        open_res["power_source"] = sampler.source

    for wk in workers:
        wk.h.graphs(False)
    roofline = measure_roofline(pool)
    # ... and every worker on the CU share it is served on: its request's solo latency there (sum over its kernel groups
    # of the profiled latency table, Sec. III-B factor (i)) against the matrix peak scaled by that share.  Whole requests,
    # every kernel and launch gap included -- context for `frac`, which is one kernel on all CUs.
    served_share = []
    for w, wk in enumerate(workers):
        t_ns = sum(beta[w][g][assign[w][g]] for g in range(wk.model.n_groups))
        cu_ns = sum(beta[w][g][assign[w][g]] * configs[assign[w][g]] for g in range(wk.model.n_groups))
        fl = sum(x[1] for x in gemm_work(wk.model, prof_batch[w]) if x is not None)
        fl += sum(4.0 * prof_batch[w] * L.w * L.w * L.c for L in wk.model.layers if L.op == wl.OP_ATTENTION)     # 4 B h S^2 d, h d = c
        cus_w = cu_ns / max(t_ns, 1)
        served_share.append({"worker": w, "model": wk.model.name, "batch": prof_batch[w], "cus": round(cus_w, 1), "solo_request_us": t_ns / 1e3,
                             "tflops": fl / max(t_ns, 1) / 1e3, "frac_of_scaled_peak": fl / max(t_ns, 1) / 1e3 / (MFMA_PEAK_TFLOPS * cus_w / 256.0)})
    roofline["served_share"] = served_share

    # ---- CPU oracle on the host cores, same models and inputs: one full forward pass per worker on the batch of its
    # last timed request.  The passes are the parity check of every worker's output (in the launch configuration that
    # was timed) and, timed, the CPU baseline.
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import forward as orc
        orc.run_model(wl.tiny_cnn(seed=0), wl.make_input(wl.tiny_cnn(seed=0), 1, dist="uniform"))     # builds / loads the library
        t_cpu, served, errs = 0.0, 0, []
        for w, wk in enumerate(workers):
            b, got = last_out[w]
            t1 = time.perf_counter()
            exp = orc.run_model(models[w], wk.x[:b])
            t_cpu += time.perf_counter() - t1
            served += b
            err = float(np.abs(got - exp).max() / (exp.max() - exp.min()))
            errs.append(err)
            log(f"worker {w} ({models[w].name}, batch {b}): GPU vs oracle err/range {err:.2e}")
            assert got.shape == exp.shape and np.isfinite(got).all() and err <= 2e-2, f"worker {w}: GPU output differs from the oracle: {err}"
        cpu = {"value": served / t_cpu, "unit": "inferences/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"one full forward pass per co-located model at its request batch ({served} inferences, {t_cpu:.1f} s), run one after another"}
        parity = {"checked": "last output of every worker of the timed run, every element", "max_err_over_range": errs, "tolerance": 2e-2}
        log(f"cpu oracle {cpu['value']:.3f} inf/s on {cpu['cores']} threads")

    for wk in workers:
        wk.h.free()
    pool.destroy()

    dts = sorted({wl.DT_NAMES[m.dtype] for m in models})
    out = {
        "metric": f"co-located inferences/s (closed loop, {n_w} workers) on 1xMI355X",
        "value": value, "unit": "inferences/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "+".join(dts), "data": "synthetic",
        "config": {"workload": WORKLOADS[cfg] + f", CU-mask pool {configs} per worker, switchMax {args.switch_max}",
                   "policy": args.policy, "inflight_per_worker": args.depth, "captured_requests": bool(args.graphs),
                   "allocation_cus": [[configs[c] for c in a] for a in assign], "switches": switches,
                   "streams_in_use_limit": 4, "switch_cost_ns": switch_cost_ns, "overlap_slope": round(slope, 4), "allocation_from": chosen,
                   "objective": args.objective, "throughput_floor": args.throughput_floor,
                   "candidate_allocations": [{"from": t[1], "allocation_cus": [_runs([configs[c] for c in a]) for a in t[2]], "switches": t[3],
                                              "trial_inferences_per_s": t[0], "trial_inferences_per_joule": t[4]} for t in trials]},
        "closed_loop": closed,
        "open_loop_poisson": open_res,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
    }
    print(json.dumps(out))
    torch.cuda.synchronize()
    for wk in workers:
        wk.h.free()
    pool.destroy()


if __name__ == "__main__":
    main()
