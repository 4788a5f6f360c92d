"""Pins for the forward-pass oracle: closed forms, invariants, brute force and an
independent fp64 library implementation of each operator.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import forward as orc

rng = np.random.default_rng(1234)


def rnd(*shape):
    return rng.standard_normal(shape)


# ---------------- convolution ---------------------------------------------------------
def test_conv_identity_kernel_returns_input():
    c, h, w = 5, 9, 7
    x = rnd(2, c, h, w)
    k = np.zeros((c, c, 3, 3), np.float32)
    for i in range(c):
        k[i, i, 1, 1] = 1.0
    y = orc.conv2d(x, k, None, stride=1, pad=1)
    assert np.array_equal(y, x)


def test_conv_all_ones_closed_form_with_borders():
    # y = Cin * (#in-bounds taps); taps along one axis at output o: overlap of [o*s-p, o*s-p+k) with [0, n)
    cin, cout, h, w, k, s, p = 3, 2, 8, 11, 3, 2, 1
    x = np.ones((1, cin, h, w))
    y = orc.conv2d(x, np.ones((cout, cin, k, k), np.float32), None, stride=s, pad=p)
    ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    assert y.shape == (1, cout, ho, wo)

    def taps(o, n):
        lo, hi = o * s - p, o * s - p + k
        return max(0, min(hi, n) - max(lo, 0))
    exp = np.array([[cin * taps(i, h) * taps(j, w) for j in range(wo)] for i in range(ho)], float)
    for co in range(cout):
        assert np.array_equal(y[0, co], exp)


def test_conv_1x1_equals_linear_equals_matmul():
    n, cin, cout, h, w = 2, 12, 7, 5, 6
    x = rnd(n, cin, h, w)
    wt = rnd(cout, cin).astype(np.float32)
    b = rnd(cout).astype(np.float32)
    y_conv = orc.conv2d(x, wt.reshape(cout, cin, 1, 1), b)
    rows = x.transpose(0, 2, 3, 1).reshape(-1, cin)
    y_lin = orc.linear(rows, wt, b)
    y_np = rows @ wt.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(y_lin, y_np, rtol=0, atol=1e-12)
    np.testing.assert_allclose(y_conv.transpose(0, 2, 3, 1).reshape(-1, cout), y_np, rtol=0, atol=1e-12)


def test_conv_brute_force_tiny():
    n, cin, cout, h, w, kh, s, p = 2, 3, 4, 5, 5, 3, 2, 1
    x = rnd(n, cin, h, w)
    wt = rnd(cout, cin, kh, kh).astype(np.float32)
    b = rnd(cout).astype(np.float32)
    y = orc.conv2d(x, wt, b, stride=s, pad=p)
    ho = (h + 2 * p - kh) // s + 1
    exp = np.zeros((n, cout, ho, ho))
    for a in range(n):
        for co in range(cout):
            for oh in range(ho):
                for ow in range(ho):
                    acc = float(b[co])
                    for ci in range(cin):
                        for i in range(kh):
                            for j in range(kh):
                                ih, iw = oh * s - p + i, ow * s - p + j
                                if 0 <= ih < h and 0 <= iw < w:
                                    acc += x[a, ci, ih, iw] * float(wt[co, ci, i, j])
                    exp[a, co, oh, ow] = acc
    np.testing.assert_allclose(y, exp, rtol=0, atol=1e-12)


@pytest.mark.parametrize("k,s,p,g", [(3, 1, 1, 1), (7, 2, 3, 1), (3, 2, 1, 4), (1, 2, 0, 1), (3, 1, 1, 8), (5, 3, 2, 2)])
def test_conv_matches_fp64_library(k, s, p, g):
    n, cin, cout, h, w = 2, 8, 16, 13, 10
    x = rnd(n, cin, h, w)
    wt = rnd(cout, cin // g, k, k).astype(np.float32)
    b = rnd(cout).astype(np.float32)
    y = orc.conv2d(x, wt, b, s, p, g)
    ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(wt).double(), torch.from_numpy(b).double(), s, p, 1, g)
    np.testing.assert_allclose(y, ref.numpy(), rtol=0, atol=1e-11)


def test_depthwise_is_grouped_conv_per_channel():
    c, h, w = 6, 7, 7
    x = rnd(1, c, h, w)
    wt = rnd(c, 1, 3, 3).astype(np.float32)
    y = orc.conv2d(x, wt, None, 1, 1, c)
    for ch in range(c):
        yc = orc.conv2d(x[:, ch:ch + 1], wt[ch:ch + 1], None, 1, 1, 1)
        np.testing.assert_allclose(y[:, ch:ch + 1], yc, rtol=0, atol=1e-13)


# ---------------- pooling -------------------------------------------------------------
@pytest.mark.parametrize("k,s,p", [(3, 2, 1), (2, 2, 0)])
def test_maxpool_brute_force_and_library(k, s, p):
    x = rnd(2, 3, 9, 8)
    y = orc.maxpool(x, k, s, p)
    ref = F.max_pool2d(torch.from_numpy(x), k, s, p).numpy()
    assert np.array_equal(y, ref)
    ho, wo = y.shape[2:]
    for oh in range(ho):
        for ow in range(wo):
            win = [x[1, 2, ih, iw] for ih in range(oh * s - p, oh * s - p + k) for iw in range(ow * s - p, ow * s - p + k)
                   if 0 <= ih < 9 and 0 <= iw < 8]
            assert y[1, 2, oh, ow] == max(win)


def test_gap_constant_and_mean():
    assert np.array_equal(orc.gap(np.full((2, 3, 4, 5), 2.5)), np.full((2, 3), 2.5))
    x = rnd(2, 3, 4, 5)
    np.testing.assert_allclose(orc.gap(x), x.mean(axis=(2, 3)), rtol=0, atol=1e-14)


# ---------------- softmax / layernorm / gelu ---------------------------------------------
def test_softmax_rows_sum_to_one_and_shift_invariant():
    x = rnd(17, 33) * 5
    y = orc.softmax(x)
    np.testing.assert_allclose(y.sum(-1), 1.0, rtol=0, atol=1e-12)
    y2 = orc.softmax(x + rnd(17, 1) * 100)
    np.testing.assert_allclose(y, y2, rtol=0, atol=1e-12)
    ref = torch.softmax(torch.from_numpy(x), -1).numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-14)
    # uniform row -> 1/width ; one dominant entry -> one-hot
    assert np.allclose(orc.softmax(np.zeros((1, 8))), 1 / 8)
    big = np.zeros((1, 8)); big[0, 3] = 800.0
    assert orc.softmax(big)[0, 3] == 1.0


def test_layernorm_moments_and_library():
    x = rnd(9, 64) * 3 + 1.5
    eps = 1e-5
    y = orc.layernorm(x, np.ones(64, np.float32), np.zeros(64, np.float32), eps)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-13)
    var = x.var(-1)
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    g = rnd(64).astype(np.float32); b = rnd(64).astype(np.float32)
    y2 = orc.layernorm(x, g, b, eps)
    ref = F.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(g).double(), torch.from_numpy(b).double(), eps)
    np.testing.assert_allclose(y2, ref.numpy(), rtol=0, atol=1e-12)
    # a constant row has zero variance: output = beta
    yc = orc.layernorm(np.full((1, 64), 7.0), g, b, eps)
    np.testing.assert_allclose(yc[0], b, atol=1e-12)


def test_activations_closed_forms():
    x = np.linspace(-8, 8, 41).reshape(1, -1)
    relu = orc.eltwise(x, None, None, wl.ACT_RELU, 1)
    relu6 = orc.eltwise(x, None, None, wl.ACT_RELU6, 1)
    gelu = orc.eltwise(x, None, None, wl.ACT_GELU, 1)
    assert np.array_equal(relu, np.maximum(x, 0))
    assert np.array_equal(relu6, np.clip(x, 0, 6))
    exp = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x[0]])
    np.testing.assert_allclose(gelu[0], exp, rtol=0, atol=1e-15)
    # Phi(1) = 0.8413447460685429...
    assert abs(orc.eltwise(np.ones((1, 1)), None, None, wl.ACT_GELU, 1)[0, 0] - 0.8413447460685429) < 1e-15
    # bias + residual are added before the activation, bias indexed by channel
    xi = rnd(2, 3, 2, 2); b = rnd(3).astype(np.float32); r = rnd(2, 3, 2, 2)
    y = orc.eltwise(xi, b, r, wl.ACT_RELU, 1)
    np.testing.assert_allclose(y, np.maximum(xi + b.astype(np.float64)[None, :, None, None] + r, 0), atol=1e-15)


# ---------------- attention / embedding ----------------------------------------------------
def test_attention_equal_keys_is_mean_of_v():
    b, s, hd, heads = 2, 7, 8, 2
    qkv = rnd(b, s, 3 * hd)
    qkv[:, :, hd:2 * hd] = rnd(1, 1, hd)          # all keys identical -> uniform attention
    y = orc.attention(qkv, heads)
    exp = np.broadcast_to(qkv[:, :, 2 * hd:].mean(1, keepdims=True), (b, s, hd))
    np.testing.assert_allclose(y, exp, rtol=0, atol=1e-13)


def test_attention_matches_fp64_library_and_numpy():
    b, s, hd, heads = 2, 11, 24, 3
    d = hd // heads
    qkv = rnd(b, s, 3 * hd)
    y = orc.attention(qkv, heads)
    q, k, v = [torch.from_numpy(qkv[:, :, i * hd:(i + 1) * hd]).reshape(b, s, heads, d).permute(0, 2, 1, 3) for i in range(3)]
    ref = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(b, s, hd).numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)
    # explicit numpy for one head
    h = 1
    qq, kk, vv = [qkv[0, :, i * hd + h * d:i * hd + (h + 1) * d] for i in range(3)]
    sc = qq @ kk.T / math.sqrt(d)
    pr = np.exp(sc - sc.max(-1, keepdims=True)); pr /= pr.sum(-1, keepdims=True)
    np.testing.assert_allclose(y[0, :, h * d:(h + 1) * d], pr @ vv, rtol=0, atol=1e-12)


def test_embed_is_sum_of_three_rows():
    v, p, hd = 50, 16, 8
    tok, pos, typ = [rnd(n, hd).astype(np.float32) for n in (v, p, 2)]
    ids = rng.integers(0, v, size=(2, 9), dtype=np.int32)
    y = orc.embed(ids, tok, pos, typ)
    for b in range(2):
        for s in range(9):
            exp = tok[ids[b, s]].astype(np.float64) + pos[s] + typ[0]
            np.testing.assert_allclose(y[b, s], exp, atol=1e-15)


# ---------------- whole-model wiring ------------------------------------------------------
def _w(m, off, *shape):
    return torch.from_numpy(m.weights[off:off + int(np.prod(shape))].reshape(shape).astype(np.float64))


def test_tiny_cnn_against_handwired_library_model():
    m = wl.tiny_cnn(seed=0)
    x = wl.make_input(m, 2, dist="uniform")
    y = orc.run_model(m, x)
    L = m.layers
    t = torch.from_numpy(x.astype(np.float64))
    t = F.relu(F.conv2d(t, _w(m, L[0].w_off, 16, 3, 3, 3), _w(m, L[0].b_off, 16), 1, 1))
    t = F.relu(F.conv2d(t, _w(m, L[1].w_off, 32, 16, 3, 3), _w(m, L[1].b_off, 32), 2, 1))
    t = t.mean((2, 3))
    t = t @ _w(m, L[3].w_off, 10, 32).T + _w(m, L[3].b_off, 10)
    assert y.shape == (2, 10)
    np.testing.assert_allclose(y, t.numpy(), rtol=0, atol=1e-12)


def test_resnet18_wiring_against_handwired_library_model():
    m = wl.resnet(18, seed=1, hw=32, n_classes=10, width=8)
    x = wl.make_input(m, 1)
    y = orc.run_model(m, x)
    assert len(m.layers) == 23 and m.n_groups == 4
    assert [m.group_of_layer.count(g) for g in range(4)] == [6, 5, 5, 7]
    # independent wiring: walk the descriptor only for parameter offsets, structure written by hand
    convs = [L for L in m.layers if L.op == wl.OP_CONV]
    it = iter(convs)

    def conv(t, cin):
        L = next(it)
        return F.conv2d(t, _w(m, L.w_off, L.c, cin, L.kh, L.kw), _w(m, L.b_off, L.c), L.stride, L.pad)
    t = torch.from_numpy(x.astype(np.float64))
    t = F.relu(conv(t, 3))
    t = F.max_pool2d(t, 3, 2, 1)
    cin = 8
    for stage in range(4):
        planes = 8 << stage
        for blk in range(2):
            sc = t
            if stage > 0 and blk == 0:
                sc = conv(t, cin)                       # 1x1 stride-2 projection
            u = F.relu(conv(t, cin))
            t = F.relu(conv(u, planes) + sc)
            cin = planes
    t = t.mean((2, 3))
    fc = m.layers[-1]
    t = t @ _w(m, fc.w_off, 10, 64).T + _w(m, fc.b_off, 10)
    np.testing.assert_allclose(y, t.numpy(), rtol=1e-12, atol=1e-10)


def test_bert_layer_wiring_against_handwired_library_model():
    hd, heads, ffn, s = 32, 4, 64, 10
    m = wl.bert(1, hd, heads, ffn, s, vocab=100, seed=4, dtype=wl.DT_F32)
    ids = wl.make_input(m, 2)
    y = orc.run_model(m, ids)
    L = m.layers
    emb = L[0]
    tok = _w(m, emb.w_off, 100, hd); pos = _w(m, emb.g_off, emb.aux1, hd); typ = _w(m, emb.be_off, 2, hd)
    t = tok[torch.from_numpy(ids).long()] + pos[:s][None] + typ[0]

    def ln(v, Lr):
        return F.layer_norm(v, (hd,), _w(m, Lr.g_off, hd), _w(m, Lr.be_off, hd), Lr.eps)

    def lin(v, Lr, k):
        return v @ _w(m, Lr.w_off, Lr.c, k).T + _w(m, Lr.b_off, Lr.c)
    t = ln(t, L[1])
    qkv = lin(t, L[2], hd)
    q, k, v = [qkv[..., i * hd:(i + 1) * hd].reshape(2, s, heads, hd // heads).permute(0, 2, 1, 3) for i in range(3)]
    a = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(2, s, hd)
    h = ln(lin(a, L[4], hd) + t, L[5])
    f = lin(F.gelu(lin(h, L[6], hd)), L[7], ffn)
    out = ln(f + h, L[8])
    assert y.shape == (2, s, hd)
    np.testing.assert_allclose(y, out.numpy(), rtol=0, atol=1e-10)


def test_vgg_flatten_order_and_mobilenet_shapes():
    m = wl.vgg16(seed=6, hw=32, width=4, fc=16, n_classes=5)
    x = wl.make_input(m, 1)
    outs = orc.run_model(m, x, keep_all=True)
    last_pool = [i for i, L in enumerate(m.layers) if L.op == wl.OP_MAXPOOL][-1]
    fc1 = m.layers[last_pool + 1]
    flat = outs[last_pool].reshape(1, -1)                  # (C,H,W) order
    k = flat.shape[1]
    exp = np.maximum(flat @ m.weights[fc1.w_off:fc1.w_off + fc1.c * k].reshape(fc1.c, k).astype(np.float64).T, 0)
    np.testing.assert_allclose(outs[last_pool + 1], exp, rtol=0, atol=1e-12)
    mb = wl.mobilenetv2(seed=7, hw=32, n_classes=10)
    assert len(mb.layers) == 54 and mb.n_groups == 7
    assert orc.run_model(mb, wl.make_input(mb, 1)).shape == (1, 10)
    r50 = wl.resnet(50, seed=3, hw=32)
    assert [r50.group_of_layer.count(g) for g in range(4)] == [12, 13, 19, 12]


def test_storage_rounding_is_exact():
    a = rng.standard_normal(1000).astype(np.float32)
    b = wl.round_to_dtype(a, wl.DT_BF16)
    assert np.array_equal(b.view(np.uint32) & 0xFFFF, np.zeros(1000, np.uint32))
    assert np.array_equal(b, torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    h = wl.round_to_dtype(a, wl.DT_F16)
    assert np.array_equal(h, torch.from_numpy(a).half().float().numpy())


def test_storage_rounded_mode_only_adds_rounding():
    m = wl.resnet(18, seed=1, hw=32, n_classes=10, width=8)
    x = wl.make_input(m, 1)
    exact = orc.run_model(m, x, keep_all=True)
    stored = orc.run_model(m, x, keep_all=True, storage_dtype=wl.DT_BF16)
    # first layer: same arithmetic, one rounding of at most 2^-9 relative
    assert np.all(np.abs(stored[0] - exact[0]) <= np.abs(exact[0]) * 2.0 ** -8 + 1e-30)
    assert np.array_equal(stored[0], wl.round_to_dtype(exact[0].astype(np.float32), wl.DT_BF16))
    assert np.abs(stored[-1] - exact[-1]).max() <= 2e-2 * (exact[-1].max() - exact[-1].min())
    assert not np.array_equal(stored[-1], exact[-1])


# ---------------- second workload family: grouped convolution, concatenation, channel shuffle ----------------
def test_grouped_conv_equals_block_diagonal_dense_conv():
    """A grouped convolution is a dense one whose weight is zero outside the diagonal blocks: pins the group
    indexing of the routine against its own dense path."""
    rng = np.random.default_rng(5)
    g, cig, cog = 4, 3, 2
    x = rng.standard_normal((2, g * cig, 6, 7))
    w = rng.standard_normal((g * cog, cig, 3, 3))
    dense = np.zeros((g * cog, g * cig, 3, 3))
    for k in range(g):
        dense[k * cog:(k + 1) * cog, k * cig:(k + 1) * cig] = w[k * cog:(k + 1) * cog]
    a = orc.conv2d(x, w, None, 2, 1, g)
    b = orc.conv2d(x, dense, None, 2, 1, 1)
    assert np.allclose(a, b, rtol=0, atol=1e-12)


def test_shuffle_is_the_index_permutation_and_inverts():
    m = wl.single_layer("shuffle", wl.DT_F32, c=12, h=2, w=3, groups=3)
    x = wl.make_input(m, 2)
    y = orc.run_model(m, x)
    n = 12 // 3
    for j in range(12):                       # written out from the definition: out j <- in (j % g) * n + j // g
        assert np.array_equal(y[:, j], x[:, (j % 3) * n + j // 3])
    # shuffling with g and then with c / g is the identity
    m2 = wl.single_layer("shuffle", wl.DT_F32, c=12, h=2, w=3, groups=4)
    assert np.array_equal(orc.run_model(m2, y.astype(np.float32)), x)
    # one group, or one channel per group, moves nothing
    for g in (1, 12):
        mi = wl.single_layer("shuffle", wl.DT_F32, c=12, h=2, w=3, groups=g)
        assert np.array_equal(orc.run_model(mi, x), x)


def test_concat_keeps_both_operands_in_order():
    m = wl.single_layer("concat", wl.DT_F32, rows=5, c0=8, c1=8)
    x = wl.make_input(m, 2)
    outs = orc.run_model(m, x, keep_all=True)
    assert outs[-1].shape == (2, 5, 16)
    assert np.array_equal(outs[-1][..., :8], x) and np.array_equal(outs[-1][..., 8:], outs[0])


def test_albert_layers_share_one_set_of_weights():
    m = wl.albert(n_layers=3, hidden=64, heads=2, ffn=128, seq=8, vocab=50, embed=32)
    lin = [L for L in m.layers if L.op == wl.OP_LINEAR][1:]              # skip the embedding projection
    per_layer = [lin[i:i + 4] for i in range(0, len(lin), 4)]
    assert len(per_layer) == 3
    for layer in per_layer[1:]:
        assert [L.w_off for L in layer] == [L.w_off for L in per_layer[0]]
    # and the blob holds one encoder layer, not three
    one = wl.albert(n_layers=1, hidden=64, heads=2, ffn=128, seq=8, vocab=50, embed=32)
    assert m.weights.size == one.weights.size
