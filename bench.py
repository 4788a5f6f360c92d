#!/usr/bin/env python3
"""Co-located inference benchmark on one MI355X.

Workload (default): two ResNet-18-style CNNs, bf16, batch 1, 3x224x224 N(0,1) inputs, He-normal weights
(seeds 1 and 2), each cut into 4 kernel groups (its stages), served by one worker thread per model on a
pre-allocated pool of CU-masked streams {32,64,128,192,256 CUs} per worker plus one shared unmasked stream.
The CU share of every group comes from the library's exact solver of the paper's allocation model, fed with
latency-vs-CU tables profiled here.

One step = one inference on every co-located model.  The timed region is exactly `--steps` steps under the
ECLIP policy with inputs resident in HBM; `value` is total inferences per second.  Around it, untimed:
the same closed loop under the two unpartitioned policies, an open-loop Poisson run (200 requests/s per
model) for p99 latency and inferences per joule, per-kernel HIP-event timings of the dominant kernel for
the roofline entry, and the CPU oracle timed on the host cores.

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

CONFIGS = [32, 64, 128, 192, 256]
HBM_PEAK_GBS = 8000.0


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
        self.dt = 1.0 / hz
        self.samples = []
        self.source = "hwmon" if self.paths else "amd-smi"
        self._stop = threading.Event()
        self._th = None

    def read(self):
        if self.paths:
            try:
                return sum(int(open(p).read()) for p in self.paths[:1]) / 1e6
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

    def _run(self):
        while not self._stop.is_set():
            v = self.read()
            if v is not None:
                self.samples.append((time.perf_counter(), v))
            self._stop.wait(self.dt)

    def start(self):
        self.samples = []
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
def conv_gemm_bytes(model, batch):
    """Algorithmic HBM bytes of every matrix-core conv/linear layer: input + weights + output (+ residual),
    2 bytes per element; im2col duplication is not traffic."""
    import workloads as wl
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
        out.append((2.0 * (n_in + n_w + n_out + (n_out if L.in1 != -2 else 0)), flops))
    return out


class Worker:
    """One model = one worker: holds the device buffers and runs closed-loop or scheduled requests."""

    def __init__(self, ec, torch, pool, model, index, depth):
        import workloads as wl
        self.model, self.index, self.depth = model, index, depth
        self.h = ec.Model(pool, model, wl.to_storage(model.weights, model.dtype), max_batch=1, max_inflight=depth)
        x = wl.make_input(model, 1)
        s = wl.to_storage(x, model.dtype)
        self.x = x
        self.d_in = torch.from_numpy(s.view(np.int16) if s.dtype == np.uint16 else s).cuda()
        self.d_out = [torch.zeros(model.out_shape(1), dtype=torch.float32, device="cuda") for _ in range(depth)]

    def closed_loop(self, n, barrier=None):
        """n inferences, up to `depth` in flight."""
        if barrier is not None:
            barrier.wait()
        q = []
        for i in range(n):
            if len(q) == self.depth:
                q.pop(0).wait()
            q.append(self.h.submit(self.d_in.data_ptr(), self.d_out[i % self.depth].data_ptr(), 1))
        for r in q:
            r.wait()

    def open_loop(self, arrivals, t_start, lat_out):
        """Serve requests at their scheduled arrival times (seconds after t_start); latency = completion - arrival."""
        for a in arrivals:
            now = time.perf_counter() - t_start
            if a > now:
                time.sleep(max(0.0, a - now - 50e-6))
                while time.perf_counter() - t_start < a:
                    pass
            self.h.submit(self.d_in.data_ptr(), self.d_out[0].data_ptr(), 1).wait()
            lat_out.append(time.perf_counter() - t_start - a)


def run_closed(workers, steps):
    bar = threading.Barrier(len(workers) + 1)
    th = [threading.Thread(target=w.closed_loop, args=(steps, bar)) for w in workers]
    [t.start() for t in th]
    bar.wait()
    t0 = time.perf_counter()
    [t.join() for t in th]
    return time.perf_counter() - t0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--depth", type=int, default=2, help="requests each worker keeps in flight")
    ap.add_argument("--window", type=float, default=10.0, help="seconds of open-loop Poisson load per policy (0 = skip)")
    ap.add_argument("--rate", type=float, default=200.0, help="Poisson arrivals per second per model")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--policy", default="eclip", choices=["eclip", "unpart_a", "unpart_b"], help="policy of the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; co-located models are independent workers and would be "
              "placed on different GPUs without any exchange step. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    import paper_2506_12598_amd as ec
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.init()
    time.sleep(0.5)
    idle_w = PowerSampler().read()          # board power before any kernel of this process has run

    models = wl.config_models(1)
    n_w = len(models)
    # pool: id 0 = shared unmasked stream; ids 1..n_w = one private unmasked stream per worker (policy
    # unpart_b); then for worker w the 5 masked streams, laid out from opposite ends of the CU range
    masks = [(None, -1)] + [(None, w) for w in range(n_w)]
    mask_id = {}
    for w in range(n_w):
        for ci, c in enumerate(CONFIGS):
            mask_id[(w, ci)] = len(masks)
            masks.append((ec.eclip_mask_layout(256, 32, n_w, w, c // 32), w))
    pool = ec.Pool(masks)
    workers = [Worker(ec, torch, pool, m, i, args.depth) for i, m in enumerate(models)]
    log(f"loaded {n_w} models, pool of {len(masks)} streams")

    # ---- latency-vs-CU tables (Sec. III-B profiling) and the allocation
    t0 = time.perf_counter()
    beta, nk, per_kernel = [], [], []
    for w, wk in enumerate(workers):
        rows, counts, pk = [], [], []
        for g in range(wk.model.n_groups):
            row = []
            for ci in range(len(CONFIGS)):
                ns = wk.h.profile_group(g, mask_id[(w, ci)], batch=1, iters=15)
                row.append(int(sum(ns)))
                if ci == len(CONFIGS) - 1:
                    pk.extend(ns)
            rows.append(row)
            counts.append(wk.h.group_size(g))
        beta.append(rows); nk.append(counts); per_kernel.append(pk)
    assign, objective, switches = ec.eclip_alloc_solve(256, CONFIGS, nk, beta, 14)
    log(f"profiled in {time.perf_counter() - t0:.1f}s; allocation {assign} switches {switches}")
    tables = {
        "eclip": [[mask_id[(w, c)] for c in assign[w]] for w in range(n_w)],
        "unpart_a": [[0] * m.n_groups for m in models],
        "unpart_b": [[1 + w] * m.n_groups for w, m in enumerate(models)],
    }

    def set_policy(name):
        for wk, t in zip(workers, tables[name]):
            wk.h.alloc_set(t)

    # ---- closed-loop throughput: the timed region
    closed = {}
    order = [p for p in ("unpart_a", "unpart_b", "eclip") if p != args.policy] + [args.policy]
    for pol in order:
        set_policy(pol)
        run_closed(workers, args.warmup)
        torch.cuda.synchronize()
        dt = run_closed(workers, args.steps)
        torch.cuda.synchronize()
        closed[pol] = {"inferences_per_s": n_w * args.steps / dt, "ms_per_step": 1e3 * dt / args.steps}
        log(f"closed loop {pol}: {closed[pol]['inferences_per_s']:.0f} inf/s")
    value = closed[args.policy]["inferences_per_s"]
    ms_per_step = closed[args.policy]["ms_per_step"]

    # ---- parity spot check in this launch configuration
    from_gpu = workers[0].d_out[0].cpu().numpy().astype(np.float64)

    # ---- open loop: Poisson arrivals, p99 latency, energy
    open_res = {}
    if args.window > 0:
        sampler = PowerSampler()
        for pol in ("unpart_a", "unpart_b", "eclip"):
            set_policy(pol)
            arr = [wl.poisson_arrivals(args.rate, args.window, i) for i in range(n_w)]
            lats = [[] for _ in workers]
            sampler.start()
            t_start = time.perf_counter() + 0.05
            th = [threading.Thread(target=wk.open_loop, args=(arr[i], t_start, lats[i])) for i, wk in enumerate(workers)]
            [t.start() for t in th]
            [t.join() for t in th]
            t_end = time.perf_counter()
            sampler.stop()
            allv = np.concatenate([np.array(l) for l in lats])
            e = sampler.energy_j(t_start, t_end)
            open_res[pol] = {
                "offered_per_s": args.rate * n_w,
                "completed": int(allv.size),
                "inferences_per_s": float(allv.size / (t_end - t_start)),
                "p50_latency_ms": float(np.percentile(allv, 50) * 1e3),
                "p99_latency_ms": float(np.percentile(allv, 99) * 1e3),
                "avg_power_w": None if e is None else e / (t_end - t_start),
                "inferences_per_joule": None if e is None else float(allv.size / e),
            }
            log(f"open loop {pol}: p99 {open_res[pol]['p99_latency_ms']:.3f} ms, "
                f"{open_res[pol]['inferences_per_joule']} inf/J")
        open_res["idle_power_w"] = idle_w
        open_res["power_source"] = sampler.source

    # ---- roofline of the dominant kernel: HIP-event timings on the stream the kernels run on.  Each layer of each
    # model is timed on that worker's unpartitioned stream (8 back-to-back launches per sample, see
    # eclip_profile_group); layers are grouped by the kernel function that runs them and the function with the
    # largest total time is reported against the roofline that bounds it at these shapes (HBM: the convolutions
    # of a batch-1 ResNet-18 have 43-230 FLOP/B, below the 315 FLOP/B ridge of the matrix cores).
    set_policy("unpart_b")
    per_kernel = {}
    for w, wk in enumerate(workers):
        ns_all = []
        for g in range(wk.model.n_groups):
            ns_all.extend(wk.h.profile_group(g, 1 + w, batch=1, iters=30))
        lb = conv_gemm_bytes(wk.model, 1)
        for li, ns in enumerate(ns_all):
            info = wk.h.kernel_info(li, 1 + w, 1)
            e = per_kernel.setdefault(info["kernel"], {"ns": 0.0, "bytes": 0.0, "flops": 0.0, "launches": 0, "layers": 0})
            e["ns"] += ns
            e["launches"] += info["launches"]
            e["layers"] += 1
            if lb[li] is not None:
                e["bytes"] += lb[li][0]
                e["flops"] += lb[li][1]
    # a layer whose K is cut over the grid runs two kernels (GEMM + slice sum): its time is attributed per launch
    dom = max((k for k in per_kernel if per_kernel[k]["bytes"] > 0),
              key=lambda k: per_kernel[k]["ns"] * per_kernel[k]["layers"] / per_kernel[k]["launches"])
    d = per_kernel[dom]
    achieved = d["bytes"] / d["ns"]          # bytes per ns = GB/s
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": dom,
                "layers_per_step": d["layers"], "launches_per_step": d["launches"], "avg_layer_us": d["ns"] / d["layers"] / 1e3,
                "avg_bytes_per_layer": d["bytes"] / d["layers"], "achieved_tflops": d["flops"] / d["ns"] / 1e3,
                "time_share_by_kernel": {k: v["ns"] / sum(x["ns"] for x in per_kernel.values()) for k, v in per_kernel.items()}}

    # ---- CPU oracle on the host cores, same models and inputs
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import forward as orc
        orc.run_model(models[0], workers[0].x)              # builds / warms the library
        t0 = time.perf_counter()
        n = 0
        exp0 = None
        while time.perf_counter() - t0 < 10.0 or n < n_w:
            y = orc.run_model(models[n % n_w], workers[n % n_w].x)
            if n == 0:
                exp0 = y
            n += 1
        dt = time.perf_counter() - t0
        cpu = {"value": n / dt, "unit": "inferences/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"{n} full forward passes of the {n_w} models (batch 1), {dt:.1f} s"}
        err = float(np.abs(from_gpu - exp0).max() / (exp0.max() - exp0.min()))
        assert err <= 2e-2, f"GPU logits differ from the oracle: {err}"
        log(f"cpu oracle {cpu['value']:.2f} inf/s on {cpu['cores']} threads; GPU vs oracle err/range {err:.2e}")

    for wk in workers:
        wk.h.free()
    pool.destroy()

    out = {
        "metric": "co-located inferences/s (closed loop, 2 workers) on 1xMI355X",
        "value": value, "unit": "inferences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "2x ResNet-18-style bf16 batch 1 3x224x224, 4 kernel groups each, CU-mask pool "
                               "{32,64,128,192,256} per worker, switchMax 14", "policy": args.policy,
                   "inflight_per_worker": args.depth, "allocation_cus": [[CONFIGS[c] for c in a] for a in assign],
                   "switches": switches},
        "closed_loop": closed,
        "open_loop_poisson": open_res,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
