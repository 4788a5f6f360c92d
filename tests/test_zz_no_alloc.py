"""eclip_submit_static (the entry point that allocates nothing) against eclip_submit, through the C ABI.

The two calls run the same kernels with the same plans; only the scratch memory differs (the library's static device
array instead of the workspace allocated at load), so the outputs must agree bit for bit.  Two calls in a row, the
second with a smaller input, so that stale partial sums of the first call sit in the shared array when the second
one runs.  The model is run so that the scratch is really used: every matrix-core layer is forced onto the LDS-tiled
kernel with K cut into slices (partial sums -> scratch -> slice-sum kernel); the kernel count of the request shows
that the slices are there."""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import forward as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2506_12598_amd as ec  # noqa: E402
from gpu_util import GpuModel, dev_input, rel_to_range  # noqa: E402


def _run(g, x, static):
    batch = x.shape[0]
    d_in = dev_input(g.model, x)
    out = torch.full(g.model.out_shape(batch), float("nan"), dtype=torch.float32, device="cuda")
    req = (g.h.submit_static if static else g.h.submit)(d_in.data_ptr(), out.data_ptr(), batch)
    _, n_kernels, _ = req.wait(timing=True)
    return out.cpu().numpy().astype(np.float64), n_kernels


def test_submit_static_matches_submit_twice_second_call_smaller():
    os.environ["ECLIP_GEMM_FORCE"] = "0,1,4"            # LDS-tiled 64 x 64 x 64 tile, K in up to 4 slices
    try:
        m = wl.resnet(18, seed=3, hw=96)
        g = GpuModel(m, max_batch=3)
        try:
            x3 = wl.make_input(m, 3)
            x1 = wl.make_input(m, 1, seed=77)
            for x in (x3, x1):                          # second call: smaller batch
                ref, n_ref = _run(g, x, static=False)
                got, n_got = _run(g, x, static=True)
                assert n_got == n_ref
                # K slices in use: more kernels than layers + input stage
                assert n_ref > len(m.layers) + 1, f"{n_ref} kernels: the K split (and with it the scratch) is not in use"
                assert np.isfinite(got).all()
                assert np.array_equal(got, ref), f"static scratch changes the result: max diff {np.abs(got - ref).max()}"
                exp = orc.run_model(m, x)
                assert rel_to_range(got, exp) <= 2e-2
        finally:
            g.free()
    finally:
        os.environ.pop("ECLIP_GEMM_FORCE", None)


def test_submit_static_rejects_a_model_beyond_the_scratch():
    # a batch-8 ResNet-18 at 224 x 224 asks for more K-slice workspace than the static array holds
    m = wl.resnet(18, seed=3)
    g = GpuModel(m, max_batch=8)
    try:
        x = wl.make_input(m, 1)
        d_in = dev_input(m, x)
        out = torch.zeros(m.out_shape(1), dtype=torch.float32, device="cuda")
        with pytest.raises(ec.EclipError) as e:
            g.h.submit_static(d_in.data_ptr(), out.data_ptr(), 1)
        assert e.value.status == ec.ELIMIT and "scratch" in e.value.message
        g.h.submit(d_in.data_ptr(), out.data_ptr(), 1).wait()      # the ordinary entry point still serves it
    finally:
        g.free()
