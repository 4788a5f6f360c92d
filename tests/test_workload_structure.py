"""Pins for the *structure* the shared generator writes (workloads/graphs.py).

Both the oracle and the library read the same layer graph, so parity between them says nothing about whether the
graph is the network its name promises: a stride in the wrong convolution of a bottleneck would pass.  These tests
pin the graphs to things outside the generator:

  * the parameter counts and multiply-accumulate counts of the published architectures (the figures commonly quoted
    for the 224 x 224 ImageNet classifiers and for the BERT encoders; normalisation layers are folded here, so their
    parameters are subtracted from the quoted totals);
  * hand-wired forward passes (structure typed out here from the architecture definitions, tensors by the library's
    fp64 routines) that walk the descriptor only for parameter offsets -- for a ResNet bottleneck network, a
    MobileNetV2 network, a VGG conv stack, a ResNeXt, a DenseNet and a ShuffleNet -- compared with the oracle's
    run of the generated graph.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import forward as orc

torch = pytest.importorskip("torch")
F = torch.nn.functional


def _w(m, off, *shape):
    n = int(np.prod(shape))
    return torch.from_numpy(m.weights[off:off + n].reshape(shape).astype(np.float64))


def _in_dims(m, L):
    if L.in0 == -1:
        return m.in_c, m.in_h, m.in_w
    P = m.layers[L.in0]
    return P.c, P.h, P.w


def count(m):
    """(weight elements of conv / linear layers counted once per distinct blob offset, multiply-accumulates per sample)."""
    seen, n_w, macs = set(), 0, 0
    for L in m.layers:
        if L.op == wl.OP_CONV:
            cin, _, _ = _in_dims(m, L)
            per_out = (cin // L.groups) * L.kh * L.kw
            macs += L.c * L.h * L.w * per_out
        elif L.op == wl.OP_LINEAR:
            cin, h, w = _in_dims(m, L)
            seq = L.kind == wl.KIND_SEQ
            per_out = cin if seq else cin * h * w
            macs += L.c * (L.w if seq else 1) * per_out
        elif L.op == wl.OP_ATTENTION:
            macs += 2 * L.w * L.w * L.c          # Q K^T and P V
            continue
        else:
            continue
        if L.w_off not in seen:
            seen.add(L.w_off)
            n_w += L.c * per_out
    return n_w, macs


# total parameters as published for the torchvision-style definitions, minus normalisation parameters (2 per
# normalised channel) and minus biases: what remains are the convolution and classifier weights
PUBLISHED = {
    # name: (builder, weights, GMACs at 224 x 224, kernels)
    "resnet18": (lambda: wl.resnet(18), 11_689_512 - 2 * 4_800 - 1_000, 1.81, 23),
    "resnet50": (lambda: wl.resnet(50), 25_557_032 - 2 * 26_560 - 1_000, 4.09, 56),
    "resnet152": (lambda: wl.resnet(152), 60_192_808 - 2 * 75_712 - 1_000, 11.51, 158),
    "vgg16": (lambda: wl.vgg16(), 138_357_544 - (2 * 64 + 2 * 128 + 3 * 256 + 6 * 512) - (4096 + 4096 + 1000), 15.47, 21),
    "mobilenetv2": (lambda: wl.mobilenetv2(), 3_504_872 - 2 * 17_056 - 1_000, 0.30, 54),
}


@pytest.mark.parametrize("name", sorted(PUBLISHED))
def test_cnn_graphs_have_the_published_parameter_and_mac_counts(name):
    build, n_weights, gmacs, n_kernels = PUBLISHED[name]
    m = build()
    n_w, macs = count(m)
    assert n_w == n_weights, f"{name}: {n_w} weights, the architecture has {n_weights}"
    assert abs(macs / 1e9 - gmacs) <= 0.006 + 0.003 * gmacs, f"{name}: {macs / 1e9:.3f} GMACs, published {gmacs}"
    assert len(m.layers) == n_kernels
    assert abs(m.flops_per_sample - 2.0 * macs) <= 1e-9 * macs       # the generator's own tally counts the same layers


def test_bert_graphs_have_the_encoder_sizes_of_the_configurations():
    # encoder weights per layer: 4 Hd^2 (Q, K, V, output) + 2 Hd FFN; flops per layer at S tokens:
    # 2 S (4 Hd^2 + 2 Hd FFN) for the linear layers + 4 S^2 Hd for the attention
    for n_layers, hd, heads, ffn, seq, gflop, mb in ((12, 768, 12, 3072, 128, 22.3, 170.0), (24, 1024, 16, 4096, 384, 986.0 / 4, 604.0)):
        m = wl.bert(n_layers, hd, heads, ffn, seq)
        n_w, macs = count(m)
        assert n_w == n_layers * (4 * hd * hd + 2 * hd * ffn)
        assert abs(n_w * 2 / 1e6 - mb) / mb < 0.01
        assert macs == n_layers * (seq * (4 * hd * hd + 2 * hd * ffn) + 2 * seq * seq * hd)
        assert abs(2 * macs / 1e9 - gflop) / gflop < 0.01
        assert len(m.layers) == 2 + 7 * n_layers                   # embedding + its LayerNorm + 7 kernels per layer
        emb = m.layers[0]
        assert emb.aux0 == 30522 and emb.c == hd


def _convs(m):
    it = iter([L for L in m.layers if L.op == wl.OP_CONV])

    def conv(t, act=None, res=None):
        L = next(it)
        cin = t.shape[1]
        y = F.conv2d(t, _w(m, L.w_off, L.c, cin // L.groups, L.kh, L.kw), _w(m, L.b_off, L.c), L.stride, L.pad, 1, L.groups)
        if res is not None:
            y = y + res
        if act == "relu":
            y = F.relu(y)
        elif act == "relu6":
            y = torch.clamp(y, 0.0, 6.0)
        return y, L
    return conv


def _head(m, t):
    fc = m.layers[-1]
    t = t.mean((2, 3))
    return t @ _w(m, fc.w_off, fc.c, t.shape[1]).T + _w(m, fc.b_off, fc.c)


def test_resnet50_bottleneck_wiring_against_handwired_model():
    """ResNet-50 (v1.5): per stage 3 / 4 / 6 / 3 bottlenecks 1x1 -> 3x3 -> 1x1 (x4 channels); the stride of a stage's first
    block sits on the 3x3 convolution and on the 1x1 projection of its shortcut; every first block projects."""
    width = 8
    m = wl.resnet(50, seed=3, hw=32, n_classes=7, width=width)
    x = wl.make_input(m, 2)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    t, L = conv(t, "relu")
    assert (L.kh, L.stride, L.pad) == (7, 2, 3)
    t = F.max_pool2d(t, 3, 2, 1)
    for stage, n in enumerate((3, 4, 6, 3)):
        planes = width << stage
        for blk in range(n):
            s = 2 if (stage > 0 and blk == 0) else 1
            sc = t
            if blk == 0:
                sc, L = conv(t)
                assert (L.kh, L.stride, L.c) == (1, s, 4 * planes)
            u, L = conv(t, "relu")
            assert (L.kh, L.stride, L.c) == (1, 1, planes)
            u, L = conv(u, "relu")
            assert (L.kh, L.stride, L.pad, L.c) == (3, s, 1, planes)
            t, L = conv(u, "relu", res=sc)
            assert (L.kh, L.stride, L.c) == (1, 1, 4 * planes)
    out = _head(m, t)
    np.testing.assert_allclose(orc.run_model(m, x), out.numpy(), rtol=1e-11, atol=1e-9)


def test_mobilenetv2_inverted_residual_wiring_against_handwired_model():
    """MobileNetV2: stem 3x3/2 -> 32; (t, c, n, s) blocks of 1x1 expand (x t, absent when t = 1) + ReLU6, depthwise 3x3
    (stride s on the first block of a row) + ReLU6, linear 1x1 projection, identity shortcut when stride 1 and equal
    channel counts; 1x1 -> 1280 + ReLU6; pool; classifier."""
    m = wl.mobilenetv2(seed=7, hw=32, n_classes=9, dtype=wl.DT_F32)
    x = wl.make_input(m, 2)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    t, L = conv(t, "relu6")
    assert (L.kh, L.stride, L.c) == (3, 2, 32)
    for tt, c, n, s in ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)):
        for i in range(n):
            stride = s if i == 0 else 1
            cin = t.shape[1]
            u = t
            if tt != 1:
                u, L = conv(u, "relu6")
                assert (L.kh, L.c, L.groups) == (1, cin * tt, 1)
            u, L = conv(u, "relu6")
            assert (L.kh, L.stride, L.pad, L.groups, L.c) == (3, stride, 1, cin * tt, cin * tt)
            t, L = conv(u, None, res=t if (stride == 1 and cin == c) else None)
            assert (L.kh, L.c, L.act) == (1, c, wl.ACT_NONE)
    t, L = conv(t, "relu6")
    assert L.c == 1280
    out = _head(m, t)
    np.testing.assert_allclose(orc.run_model(m, x), out.numpy(), rtol=1e-11, atol=1e-9)


def test_vgg16_conv_stack_wiring_against_handwired_model():
    m = wl.vgg16(seed=6, hw=32, width=4, fc=16, n_classes=5)
    x = wl.make_input(m, 1)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    for mult, n in ((1, 2), (2, 2), (4, 3), (8, 3), (8, 3)):
        for _ in range(n):
            t, L = conv(t, "relu")
            assert (L.kh, L.stride, L.pad, L.c) == (3, 1, 1, 4 * mult)
        t = F.max_pool2d(t, 2, 2)
    t = t.reshape(1, -1)
    for i, L in enumerate(m.layers[-3:]):
        t = t @ _w(m, L.w_off, L.c, t.shape[1]).T + _w(m, L.b_off, L.c)
        if i < 2:
            t = F.relu(t)
    np.testing.assert_allclose(orc.run_model(m, x), t.numpy(), rtol=1e-11, atol=1e-9)


def test_resnext_grouped_bottleneck_wiring_against_handwired_model():
    m = wl.resnext(reps=(2, 2, 1, 1), groups=4, width_per_group=2, seed=23, hw=32, n_classes=6, res_scale=0.5)
    x = wl.make_input(m, 1)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    t, _ = conv(t, "relu")
    t = F.max_pool2d(t, 3, 2, 1)
    for stage, n in enumerate((2, 2, 1, 1)):
        inner, cout = (4 * 2) << stage, 256 << stage
        for blk in range(n):
            s = 2 if (stage > 0 and blk == 0) else 1
            sc = t
            if blk == 0:
                sc, L = conv(t)
                assert (L.kh, L.stride, L.c) == (1, s, cout)
            u, L = conv(t, "relu")
            assert (L.kh, L.c, L.groups) == (1, inner, 1)
            u, L = conv(u, "relu")
            assert (L.kh, L.stride, L.groups, L.c) == (3, s, 4, inner)
            t, L = conv(u, "relu", res=sc)
            assert (L.kh, L.c) == (1, cout)
    np.testing.assert_allclose(orc.run_model(m, x), _head(m, t).numpy(), rtol=1e-11, atol=1e-9)


def test_densenet_concatenation_wiring_against_handwired_model():
    growth, bott = 8, 4
    m = wl.densenet(blocks=(2, 3, 2), growth=growth, seed=22, hw=32, n_classes=5, bottleneck=bott)
    x = wl.make_input(m, 1)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    t, L = conv(t, "relu")
    assert L.c == 2 * growth
    t = F.max_pool2d(t, 3, 2, 1)
    for bi, n in enumerate((2, 3, 2)):
        for _ in range(n):
            u, L = conv(t, "relu")
            assert (L.kh, L.c) == (1, bott * growth)
            u, L = conv(u, "relu")
            assert (L.kh, L.pad, L.c) == (3, 1, growth)
            t = torch.cat([t, u], 1)                      # input first, new features after it
        if bi < 2:
            t, L = conv(t, "relu")
            assert (L.kh, L.c) == (1, t.shape[1])
            t = F.max_pool2d(t, 2, 2)
    np.testing.assert_allclose(orc.run_model(m, x), _head(m, t).numpy(), rtol=1e-11, atol=1e-9)


def test_shufflenet_unit_wiring_against_handwired_model():
    g = 2
    m = wl.shufflenet(groups=g, reps=(2, 2, 1), base=32, seed=24, hw=32, n_classes=5)
    x = wl.make_input(m, 1)
    conv = _convs(m)
    t = torch.from_numpy(x.astype(np.float64))
    t, _ = conv(t, "relu")
    t = F.max_pool2d(t, 3, 2, 1)
    for stage, n in enumerate((2, 2, 1)):
        cout = 32 << stage
        for blk in range(n):
            s = 2 if blk == 0 else 1
            cin = t.shape[1]
            sc = t
            if not (s == 1 and cin == cout):
                sc, L = conv(t)
                assert (L.kh, L.stride, L.c) == (1, s, cout)
            u, L = conv(t, "relu")
            assert (L.kh, L.c, L.groups) == (1, cout // 4, 1 if cin % g else g)
            b_, c_, h_, w_ = u.shape
            u = u.reshape(b_, g, c_ // g, h_, w_).transpose(1, 2).reshape(b_, c_, h_, w_)       # channel shuffle
            u, L = conv(u)
            assert (L.kh, L.stride, L.groups) == (3, s, cout // 4)
            t, L = conv(u, "relu", res=sc)
            assert (L.kh, L.groups, L.c) == (1, g, cout)
    np.testing.assert_allclose(orc.run_model(m, x), _head(m, t).numpy(), rtol=1e-11, atol=1e-9)
