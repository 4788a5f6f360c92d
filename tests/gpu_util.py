"""Helpers for the GPU parity tests: run a workloads.Model through the C ABI and through the oracle."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
import paper_2506_12598_amd as ec

_pool = None


def shared_pool():
    """One unmasked stream (id 0) plus CU-masked streams of 32/64/128/192/256 CUs (ids 1..5)."""
    global _pool
    if _pool is None:
        masks = [(None, -1)]
        for take in (1, 2, 4, 6, 8):
            masks.append((ec.eclip_mask_layout(256, 32, 2, 0, take), 0))
        _pool = ec.Pool(masks)
    return _pool


def dev_input(model, x: np.ndarray) -> torch.Tensor:
    if model.in_kind == wl.IN_TOKENS:
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    s = wl.to_storage(x, model.dtype)
    if s.dtype == np.uint16:
        s = s.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(s)).cuda()


class GpuModel:
    def __init__(self, model, max_batch=1, pool=None, max_inflight=4):
        self.model = model
        self.pool = pool or shared_pool()
        self.h = ec.Model(self.pool, model, wl.to_storage(model.weights, model.dtype), max_batch, max_inflight)
        self.h.alloc_set([0] * model.n_groups)

    def run(self, x: np.ndarray, table=None, timing=False):
        if table is not None:
            self.h.alloc_set(table)
        batch = x.shape[0]
        self.h.timing(timing)
        d_in = dev_input(self.model, x)
        out = torch.full(self.model.out_shape(batch), float("nan"), dtype=torch.float32, device="cuda")
        req = self.h.submit(d_in.data_ptr(), out.data_ptr(), batch)
        t = req.wait(timing=timing)
        res = out.cpu().numpy().astype(np.float64)
        return (res, t) if timing else res

    def free(self):
        self.h.free()


def run_gpu(model, x, **kw):
    g = GpuModel(model, max_batch=x.shape[0], **kw)
    try:
        return g.run(x)
    finally:
        g.free()


def rel_to_range(got, exp):
    rng = float(exp.max() - exp.min())
    return float(np.abs(got - exp).max()) / (rng if rng > 0 else 1.0)
