"""GPU parity at the configurations' full sizes, through the same entry points and launch configuration the
benchmark uses (batch, dtype, kernel groups on masked streams).  The oracle's whole forward pass is affordable at
these sizes on the host cores (0.3 - 20 s each), so every output element is compared."""
import numpy as np
import pytest

import workloads as wl
from oracle import forward as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import GpuModel, rel_to_range  # noqa: E402


def full_check(model, batch, table, tol=2e-2):
    x = wl.make_input(model, batch)
    g = GpuModel(model, max_batch=batch)
    try:
        got = g.run(x, table=table)
    finally:
        g.free()
    exp = orc.run_model(model, x)
    assert got.shape == exp.shape and np.isfinite(got).all()
    err = rel_to_range(got, exp)
    assert err <= tol, f"{model.name}: err/range {err}"
    return err


def test_config3_resnet50_bf16_and_bert_base_fp16():
    r50, bert = wl.config_models(2)
    assert len(r50.layers) == 56 and [r50.group_of_layer.count(g) for g in range(4)] == [12, 13, 19, 12]
    full_check(r50, 1, [3, 2, 4, 1])
    assert bert.n_groups == 4 and bert.layers[-1].c == 768 and bert.in_w == 128
    full_check(bert, 1, [2, 5, 3, 0])


def test_config4_vgg16_and_mobilenetv2_batch_range():
    _, vgg, mbv2, _ = wl.config_models(3)
    assert vgg.n_groups == 6 and mbv2.n_groups == 7 and len(mbv2.layers) == 54
    full_check(vgg, 2, [5, 5, 4, 3, 2, 1])
    full_check(mbv2, 8, [1, 2, 3, 4, 5, 0, 3])


def test_config5_resnet152_batch8_bf16():
    m = wl.config_models(4)[3]
    assert [m.group_of_layer.count(g) for g in range(4)] == [12, 25, 109, 12]
    full_check(m, 8, [5, 4, 5, 3])


@pytest.mark.parametrize("worker", [0, 1, 2])
def test_config5_bert_large_all_24_layers_seq384_batch4_bf16(worker):
    # the three encoders of the stress configuration as the benchmark loads them (24 layers, hidden 1024, 16 heads, FFN 4096,
    # S = 384, batch 4, seeds 9-11, 8 kernel groups of 3 layers), each on a table of masked streams that switches at group
    # boundaries; the oracle's full forward pass takes about 16 s per encoder on the host cores
    m = wl.bert(24, 1024, 16, 4096, 384, seed=9 + worker, dtype=wl.DT_BF16)       # = wl.config_models(4)[worker]
    assert len(m.layers) == 2 + 7 * 24 and m.n_groups == 8 and m.in_w == 384 and m.layers[-1].c == 1024
    full_check(m, 4, [[3, 3, 5, 5, 4, 4, 3, 3], [5, 4, 3, 2, 1, 2, 3, 4], [2, 2, 2, 2, 5, 5, 5, 5]][worker])


def test_config4_resnet50_vgg16_and_bert_base_at_batch_8():
    # configuration 4 draws the batch of every request from 1..8: the three models that the other tests run at batch 1 or 2,
    # at the top of that range and at full size
    r50, vgg, _, bert = wl.config_models(3)
    full_check(r50, 8, [4, 3, 5, 2])
    full_check(vgg, 8, [5, 4, 5, 3, 4, 2])
    full_check(bert, 8, [3, 5, 4, 1])


def test_second_family_resnext50_and_shufflenet_full_size():
    rx, sh = wl.config_models(6)
    assert sum(1 for L in rx.layers if L.op == wl.OP_CONV and 1 < L.groups < L.c) == 16       # grouped 3x3 convolutions
    assert sum(1 for L in sh.layers if L.op == wl.OP_SHUFFLE) == 16
    full_check(rx, 1, [3, 2, 4, 1])
    full_check(sh, 1, [1, 3, 5])


def test_second_family_albert_base_and_densenet121_full_size():
    al, dn = wl.config_models(5)
    assert sum(1 for L in dn.layers if L.op == wl.OP_CONCAT) == 58 and dn.n_groups == 4
    full_check(al, 1, [2, 5, 3, 0])
    full_check(dn, 1, [4, 2, 5, 3])
