"""ctypes binding of libeclip.so: argument marshalling only, names as in include/eclip.h.

Every step of the inference path runs inside the library's HIP kernels; there is no Python or
CPU fallback.  Importing this module raises if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeclip.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE, ETIMEOUT, ELIMIT = range(7)
STATUS_NAMES = ["OK", "EINVAL", "ENOMEM", "EHIP", "ESTATE", "ETIMEOUT", "ELIMIT"]
OVERLAP_EXCESS, OVERLAP_LITERAL, OVERLAP_TABLE = range(3)
NO_TIMEOUT = 2 ** 64 - 1


class EclipError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 7 else status}: {message}")
        self.status = status
        self.message = message


class eclip_mask(C.Structure):
    _fields_ = [("words", C.POINTER(C.c_uint32)), ("n_words", C.c_uint32), ("owner", C.c_int32)]


class eclip_layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "in0", "in1", "kind", "c", "h", "w", "kh", "kw", "stride", "pad",
                                         "groups", "act", "heads")] + \
               [(n, C.c_int64) for n in ("w_off", "b_off", "g_off", "be_off")] + \
               [("eps", C.c_float), ("aux0", C.c_int32), ("aux1", C.c_int32)]


class eclip_model_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("in_kind", C.c_int32), ("in_c", C.c_int32), ("in_h", C.c_int32),
                ("in_w", C.c_int32), ("layers", C.POINTER(eclip_layer)), ("n_layers", C.c_uint32),
                ("group_of_layer", C.POINTER(C.c_uint32)), ("n_groups", C.c_uint32), ("max_batch", C.c_uint32),
                ("max_inflight", C.c_uint32)]


class eclip_timing(C.Structure):
    _fields_ = [("gpu_ns", C.c_uint64), ("n_kernels", C.c_uint32), ("n_switches", C.c_uint32)]


class eclip_kernel_info(C.Structure):
    _fields_ = [("kernel", C.c_char * 48), ("launches", C.c_uint32), ("workgroups", C.c_uint32), ("threads", C.c_uint32),
                ("tile_m", C.c_uint32), ("tile_n", C.c_uint32), ("k_splits", C.c_uint32), ("m", C.c_uint64),
                ("n", C.c_uint64), ("k", C.c_uint64)]


class eclip_u128(C.Structure):
    _fields_ = [("lo", C.c_uint64), ("hi", C.c_uint64)]


class eclip_alloc_problem(C.Structure):
    _fields_ = [("total_cus", C.c_uint32), ("configs", C.POINTER(C.c_uint32)), ("n_configs", C.c_uint32),
                ("n_workers", C.c_uint32), ("units_of_worker", C.POINTER(C.c_uint32)),
                ("n_kernels", C.POINTER(C.c_uint32)), ("beta", C.POINTER(C.c_uint64)), ("switch_max", C.c_uint32),
                ("overlap_mode", C.c_uint32), ("alpha_ppm", C.POINTER(C.c_uint64)), ("n_alpha", C.c_uint32),
                ("granule", C.c_uint32), ("max_configs", C.c_uint32), ("switch_cost_ns", C.c_uint64),
                ("max_configs_of_worker", C.POINTER(C.c_uint32))]


EXPORTS = {
    "eclip_last_error": (C.c_char_p, []),
    "eclip_pool_create": (C.c_int, [C.c_int, C.POINTER(eclip_mask), C.c_uint32, C.POINTER(C.c_void_p)]),
    "eclip_pool_stream": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p), C.POINTER(C.c_uint32)]),
    "eclip_pool_device_cus": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "eclip_pool_destroy": (C.c_int, [C.c_void_p]),
    "eclip_pool_pipe": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32)]),
    "eclip_bench_streams": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.c_uint32, C.c_uint32, C.POINTER(C.c_double)]),
    "eclip_model_rebind": (C.c_int, [C.c_void_p, C.c_void_p]),
    "eclip_mask_layout": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                    C.POINTER(C.c_uint32), C.c_uint32]),
    "eclip_pool_probe": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32)]),
    "eclip_pool_probe_graph": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32)]),
    "eclip_model_load": (C.c_int, [C.c_void_p, C.POINTER(eclip_model_desc), C.c_void_p, C.c_size_t, C.c_int,
                                   C.POINTER(C.c_void_p)]),
    "eclip_model_free": (C.c_int, [C.c_void_p]),
    "eclip_alloc_set": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.c_uint32]),
    "eclip_model_switches": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "eclip_model_group_size": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32)]),
    "eclip_model_kernel_info": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(eclip_kernel_info)]),
    "eclip_submit": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p)]),
    "eclip_submit_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p)]),
    "eclip_model_timing": (C.c_int, [C.c_void_p, C.c_int]),
    "eclip_model_graphs": (C.c_int, [C.c_void_p, C.c_int]),
    "eclip_model_tune": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32)]),
    "eclip_profile_group_served": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                             C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]),
    "eclip_wait": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(eclip_timing)]),
    "eclip_profile_group": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                      C.POINTER(C.c_uint64)]),
    "eclip_alloc_solve": (C.c_int, [C.POINTER(eclip_alloc_problem), C.POINTER(C.c_uint32), C.POINTER(eclip_u128),
                                    C.POINTER(C.c_uint32)]),
    "eclip_alloc_model_wise": (C.c_int, [C.POINTER(eclip_alloc_problem), C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32),
                                         C.POINTER(C.c_uint32)]),
    "eclip_alloc_kernel_wise": (C.c_int, [C.POINTER(eclip_alloc_problem), C.c_uint32, C.POINTER(C.c_uint32),
                                          C.POINTER(C.c_uint32)]),
    "eclip_bench_switch": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(C.c_double),
                                     C.POINTER(C.c_double), C.POINTER(C.c_double)]),
}

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_12598_amd.build` "
                      "(there is no fallback path)")
lib = C.CDLL(LIB_PATH)
for _name, (_res, _args) in EXPORTS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def last_error() -> str:
    return lib.eclip_last_error().decode()


def check(status: int) -> None:
    if status != OK:
        raise EclipError(status, last_error())


def _u32(seq) -> "C.Array":
    return (C.c_uint32 * len(seq))(*[int(v) for v in seq])


# ---- pool ---------------------------------------------------------------------------------------
def eclip_mask_layout(total_cus: int, granule: int, n_workers: int, worker: int, take: int,
                      stripe: int = 0) -> List[int]:
    n_words = (total_cus + 31) // 32
    out = (C.c_uint32 * n_words)()
    check(lib.eclip_mask_layout(total_cus, granule, n_workers, worker, take, stripe, out, n_words))
    return list(out)


def mask_bits(words: Sequence[int]) -> List[int]:
    return [i * 32 + b for i, w in enumerate(words) for b in range(32) if (w >> b) & 1]


def words_of_bits(bits: Sequence[int], n_words: int) -> List[int]:
    w = [0] * n_words
    for b in bits:
        w[b // 32] |= 1 << (b % 32)
    return w


class Pool:
    """eclip_pool_*: `masks` is a list of (words or None for an unmasked stream, owner)."""

    def __init__(self, masks: Sequence[Tuple[Optional[Sequence[int]], int]], device: int = 0):
        self._keep = []
        arr = (eclip_mask * len(masks))()
        for i, (words, owner) in enumerate(masks):
            if words is None:
                arr[i].words, arr[i].n_words = None, 0
            else:
                buf = _u32(words)
                self._keep.append(buf)
                arr[i].words, arr[i].n_words = C.cast(buf, C.POINTER(C.c_uint32)), len(words)
            arr[i].owner = owner
        self.handle = C.c_void_p()
        check(lib.eclip_pool_create(device, arr, len(masks), C.byref(self.handle)))
        self.n_masks = len(masks)

    def stream(self, mask_id: int) -> Tuple[int, int]:
        s, n = C.c_void_p(), C.c_uint32()
        check(lib.eclip_pool_stream(self.handle, mask_id, C.byref(s), C.byref(n)))
        return s.value, n.value

    def device_cus(self) -> int:
        n = C.c_uint32()
        check(lib.eclip_pool_device_cus(self.handle, C.byref(n)))
        return n.value

    def pipe(self, mask_id: int) -> int:
        n = C.c_uint32()
        check(lib.eclip_pool_pipe(self.handle, mask_id, C.byref(n)))
        return n.value

    def bench_streams(self, mask_ids: Sequence[int], iters: int) -> float:
        out = C.c_double()
        check(lib.eclip_bench_streams(self.handle, _u32(mask_ids), len(mask_ids), iters, C.byref(out)))
        return out.value

    def probe(self, mask_id: int, n_blocks: int) -> np.ndarray:
        out = np.zeros(n_blocks, np.uint32)
        check(lib.eclip_pool_probe(self.handle, mask_id, n_blocks, out.ctypes.data_as(C.POINTER(C.c_uint32))))
        return out

    def probe_graph(self, mask_id: int, n_blocks: int) -> np.ndarray:
        out = np.zeros(n_blocks, np.uint32)
        check(lib.eclip_pool_probe_graph(self.handle, mask_id, n_blocks, out.ctypes.data_as(C.POINTER(C.c_uint32))))
        return out

    def bench_switch(self, mask_a: int, mask_b: int, iters: int, with_create: bool = True):
        a, b, c = C.c_double(), C.c_double(), C.c_double()
        check(lib.eclip_bench_switch(self.handle, mask_a, mask_b, iters, C.byref(a), C.byref(b),
                                     C.byref(c) if with_create else None))
        return a.value, b.value, (c.value if with_create else None)

    def destroy(self):
        if self.handle:
            check(lib.eclip_pool_destroy(self.handle))
            self.handle = C.c_void_p()


# ---- model ---------------------------------------------------------------------------------------
def make_desc(model, max_batch: int, max_inflight: int):
    """Marshal a workloads.Model into an eclip_model_desc (returns desc and the arrays it points to)."""
    layers = (eclip_layer * len(model.layers))()
    for i, L in enumerate(model.layers):
        e = layers[i]
        for f in ("op", "in0", "in1", "kind", "c", "h", "w", "kh", "kw", "stride", "pad", "groups", "act", "heads",
                  "w_off", "b_off", "g_off", "be_off", "aux0", "aux1"):
            setattr(e, f, int(getattr(L, f)))
        e.eps = float(L.eps)
    groups = _u32(model.group_of_layer)
    d = eclip_model_desc(model.dtype, model.in_kind, model.in_c, model.in_h, model.in_w, layers, len(model.layers),
                         groups, model.n_groups, max_batch, max_inflight)
    return d, (layers, groups)


class Request:
    def __init__(self, handle):
        self.handle = handle

    def wait(self, timeout_ns: int = NO_TIMEOUT, timing: bool = False):
        t = eclip_timing()
        check(lib.eclip_wait(self.handle, timeout_ns, C.byref(t) if timing else None))
        return (t.gpu_ns, t.n_kernels, t.n_switches) if timing else None


class Model:
    """eclip_model_*: `storage` is the weight blob in the model dtype (numpy float32 / uint16 bits / float16)."""

    def __init__(self, pool: Pool, model, storage: np.ndarray, max_batch: int = 1, max_inflight: int = 4):
        self.pool = pool
        desc, keep = make_desc(model, max_batch, max_inflight)
        storage = np.ascontiguousarray(storage)
        self.handle = C.c_void_p()
        check(lib.eclip_model_load(pool.handle if pool is not None else None, C.byref(desc),
                                   storage.ctypes.data_as(C.c_void_p), storage.nbytes, 0, C.byref(self.handle)))
        self.n_groups = model.n_groups

    def rebind(self, pool: "Pool"):
        check(lib.eclip_model_rebind(self.handle, pool.handle))
        self.pool = pool

    def alloc_set(self, mask_id_of_group: Sequence[int]):
        check(lib.eclip_alloc_set(self.handle, _u32(mask_id_of_group), len(mask_id_of_group)))

    def switches(self) -> int:
        n = C.c_uint32()
        check(lib.eclip_model_switches(self.handle, C.byref(n)))
        return n.value

    def group_size(self, group: int) -> int:
        n = C.c_uint32()
        check(lib.eclip_model_group_size(self.handle, group, C.byref(n)))
        return n.value

    def kernel_info(self, layer: int, mask_id: int, batch: int = 1) -> dict:
        k = eclip_kernel_info()
        check(lib.eclip_model_kernel_info(self.handle, layer, mask_id, batch, C.byref(k)))
        return {"kernel": k.kernel.decode(), "launches": k.launches, "workgroups": k.workgroups, "threads": k.threads,
                "tile": (k.tile_m, k.tile_n), "k_splits": k.k_splits, "mnk": (k.m, k.n, k.k)}

    def submit(self, d_in: int, d_out: int, batch: int) -> Request:
        """d_in / d_out are device addresses (e.g. torch tensor .data_ptr())."""
        r = C.c_void_p()
        check(lib.eclip_submit(self.handle, C.c_void_p(d_in), C.c_void_p(d_out), batch, C.byref(r)))
        return Request(r)

    def submit_static(self, d_in: int, d_out: int, batch: int) -> Request:
        r = C.c_void_p()
        check(lib.eclip_submit_static(self.handle, C.c_void_p(d_in), C.c_void_p(d_out), batch, C.byref(r)))
        return Request(r)

    def graphs(self, enable: bool):
        check(lib.eclip_model_graphs(self.handle, 1 if enable else 0))

    def timing(self, enable: bool):
        check(lib.eclip_model_timing(self.handle, 1 if enable else 0))

    def tune(self, mask_id: int, batch: int = 1, iters: int = 2) -> int:
        """Time every candidate plan of every GEMM problem on pool entry `mask_id`; returns the number of problems timed."""
        n = C.c_uint32()
        check(lib.eclip_model_tune(self.handle, mask_id, batch, iters, C.byref(n)))
        return n.value

    def profile_group_served(self, group: int, mask_id: int, batch: int = 1, iters: int = 20) -> Tuple[int, int]:
        """(group latency in ns as served, kernels launched per pass)."""
        ns, n = C.c_uint64(), C.c_uint32()
        check(lib.eclip_profile_group_served(self.handle, group, mask_id, batch, iters, C.byref(ns), C.byref(n)))
        return ns.value, n.value

    def profile_group(self, group: int, mask_id: int, batch: int = 1, iters: int = 20) -> List[int]:
        n = self.group_size(group)
        out = (C.c_uint64 * n)()
        check(lib.eclip_profile_group(self.handle, group, mask_id, batch, iters, out))
        return list(out)

    def free(self):
        if self.handle:
            check(lib.eclip_model_free(self.handle))
            self.handle = C.c_void_p()


# ---- allocator -------------------------------------------------------------------------------------
def eclip_alloc_solve(total_cus: int, configs: Sequence[int], n_kernels: Sequence[Sequence[int]],
                      beta: Sequence[Sequence[Sequence[int]]], switch_max: int, overlap_mode: int = OVERLAP_EXCESS,
                      alpha_ppm: Optional[Sequence[int]] = None, granule: int = 1, max_configs: int = 0,
                      switch_cost_ns: int = 0, max_configs_of_worker: Optional[Sequence[int]] = None):
    """n_kernels[w][g], beta[w][g][c] -> (cfg_idx[w][g], objective:int, switches[w])."""
    units = [len(x) for x in n_kernels]
    flat_n = [v for w in n_kernels for v in w]
    flat_b = [v for w in beta for row in w for v in row]
    cfg = _u32(configs)
    uo = _u32(units)
    nk = _u32(flat_n)
    bb = (C.c_uint64 * len(flat_b))(*[int(v) for v in flat_b])
    ap = (C.c_uint64 * len(alpha_ppm))(*[int(v) for v in alpha_ppm]) if alpha_ppm else None
    mw = _u32(max_configs_of_worker) if max_configs_of_worker is not None else None
    p = eclip_alloc_problem(total_cus, cfg, len(configs), len(units), uo, nk, bb, switch_max, overlap_mode,
                            ap, len(alpha_ppm) if alpha_ppm else 0, granule, max_configs, switch_cost_ns, mw)
    out = (C.c_uint32 * max(1, sum(units)))()
    obj = eclip_u128()
    sw = (C.c_uint32 * max(1, len(units)))()
    check(lib.eclip_alloc_solve(C.byref(p), out, C.byref(obj), sw))
    res, pos = [], 0
    for g in units:
        res.append(list(out[pos:pos + g]))
        pos += g
    return res, (obj.hi << 64) | obj.lo, list(sw[:len(units)])


def _tables_problem(configs, beta):
    units = [len(x) for x in beta]
    flat_b = [v for w in beta for row in w for v in row]
    cfg, uo = _u32(configs), _u32(units)
    bb = (C.c_uint64 * len(flat_b))(*[int(v) for v in flat_b])
    p = eclip_alloc_problem(0, cfg, len(configs), len(units), uo, None, bb, 0, 0, None, 0, 0, 0, 0, None)
    return p, units, (cfg, uo, bb)


def _split(out, sw, units):
    res, pos = [], 0
    for g in units:
        res.append(list(out[pos:pos + g]))
        pos += g
    return res, list(sw[:len(units)])


def eclip_alloc_model_wise(configs: Sequence[int], beta: Sequence[Sequence[Sequence[int]]], slo_num: int = 3, slo_den: int = 1):
    """beta[w][g][c] -> (cfg_idx[w][g], switches[w]): one configuration per worker."""
    p, units, _keep = _tables_problem(configs, beta)
    out = (C.c_uint32 * max(1, sum(units)))()
    sw = (C.c_uint32 * max(1, len(units)))()
    check(lib.eclip_alloc_model_wise(C.byref(p), slo_num, slo_den, out, sw))
    return _split(out, sw, units)


def eclip_alloc_kernel_wise(configs: Sequence[int], beta: Sequence[Sequence[Sequence[int]]], tol_pct: int = 5):
    """beta[w][g][c] -> (cfg_idx[w][g], switches[w]): every unit at its own minimum-CU threshold."""
    p, units, _keep = _tables_problem(configs, beta)
    out = (C.c_uint32 * max(1, sum(units)))()
    sw = (C.c_uint32 * max(1, len(units)))()
    check(lib.eclip_alloc_kernel_wise(C.byref(p), tol_pct, out, sw))
    return _split(out, sw, units)
