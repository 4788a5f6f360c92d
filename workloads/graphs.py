"""Seeded synthetic workloads: layer-graph descriptors, weights and inputs.

This module is the only thing the CPU oracle and the GPU library have in
common.  It holds no network arithmetic: it draws random numbers, rounds them
to the storage dtype, and writes the *description* of each network (a flat
layer list in execution order).  Whoever consumes a `Model` must implement the
layer semantics itself.

Layer semantics (what a consumer has to compute), logical layouts:
  IMAGE tensors are [B, C, H, W]; SEQ tensors are [B, S, Hd] (stored in the
  descriptor as c=Hd, h=1, w=S); VEC tensors are [B, n] (c=n, h=w=1).

  CONV       y = act(conv2d(x, W[cout, cin/groups, kh, kw], stride, pad, groups) + b + in1)
  LINEAR     y = act(x . W[n, k]^T + b + in1); x is flattened per sample
             (C,H,W order) when it is an IMAGE, applied per token when it is a SEQ
  MAXPOOL    window kh x kw, stride, pad with -inf
  GAP        mean over H*W  -> VEC
  LAYERNORM  over the last axis of (x + in1), biased variance, gamma/beta
  SOFTMAX    over the last axis (c) of x
  ATTENTION  x = [B,S,3*Hd] laid out [q | k | v], each head-major; per head
             softmax(q k^T / sqrt(d)) v  -> [B,S,Hd]
  EMBED      x = int32 token ids [B,S]; y = tok[id] + pos[s] + typ[0]
  ELTWISE    y = act(x + b + in1)
  CONCAT     y = [x | in1] along the channel axis
  SHUFFLE    channel shuffle: channels viewed as (groups, c/groups), transposed, flattened

The co-location configurations these stand in for are the paper's workload
mixes (Sec. IV-A): a CNN classifier family and a transformer-encoder family,
2-4 workers per GPU.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

# ---- enums shared (by value) with the C ABI ---------------------------------
OP_CONV, OP_LINEAR, OP_MAXPOOL, OP_GAP, OP_LAYERNORM, OP_SOFTMAX, OP_ATTENTION, OP_EMBED, OP_ELTWISE, OP_CONCAT, OP_SHUFFLE = \
    range(1, 12)
ACT_NONE, ACT_RELU, ACT_RELU6, ACT_GELU = range(4)
DT_F32, DT_BF16, DT_F16 = range(3)
KIND_IMAGE, KIND_SEQ, KIND_VEC = range(3)
IN_IMAGE, IN_TOKENS, IN_SEQ, IN_VEC = range(4)

OP_NAMES = {OP_CONV: "conv", OP_LINEAR: "linear", OP_MAXPOOL: "maxpool", OP_GAP: "gap",
            OP_LAYERNORM: "layernorm", OP_SOFTMAX: "softmax", OP_ATTENTION: "attention",
            OP_EMBED: "embed", OP_ELTWISE: "eltwise", OP_CONCAT: "concat", OP_SHUFFLE: "shuffle"}
DT_NAMES = {DT_F32: "f32", DT_BF16: "bf16", DT_F16: "f16"}


@dataclass
class Layer:
    op: int
    in0: int = -1            # index of an earlier layer, or -1 = model input
    in1: int = -2            # residual / second operand; -2 = none
    kind: int = KIND_IMAGE   # kind of the output tensor
    c: int = 0               # output dims (see module docstring)
    h: int = 1
    w: int = 1
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1
    act: int = ACT_NONE
    heads: int = 0
    w_off: int = -1          # element offsets into the weight blob (-1 = absent)
    b_off: int = -1
    g_off: int = -1          # LN gamma / EMBED position table
    be_off: int = -1         # LN beta  / EMBED type table
    eps: float = 0.0
    aux0: int = 0            # EMBED: vocabulary size
    aux1: int = 0            # EMBED: number of positions


@dataclass
class Model:
    name: str
    dtype: int
    in_kind: int
    in_c: int
    in_h: int
    in_w: int
    layers: List[Layer]
    weights: np.ndarray                  # float32 values, each exactly representable in `dtype`
    group_of_layer: List[int]
    n_groups: int
    seed: int = 0
    flops_per_sample: float = 0.0        # 2*MACs of conv/linear/attention layers

    def in_shape(self, batch: int) -> Tuple[int, ...]:
        if self.in_kind == IN_IMAGE:
            return (batch, self.in_c, self.in_h, self.in_w)
        if self.in_kind == IN_TOKENS:
            return (batch, self.in_w)
        if self.in_kind == IN_SEQ:
            return (batch, self.in_w, self.in_c)
        return (batch, self.in_c)

    def out_shape(self, batch: int) -> Tuple[int, ...]:
        L = self.layers[-1]
        if L.kind == KIND_IMAGE:
            return (batch, L.c, L.h, L.w)
        if L.kind == KIND_SEQ:
            return (batch, L.w, L.c)
        return (batch, L.c)


# ---- rounding to the storage dtype (input preparation only) ------------------
def round_to_dtype(a: np.ndarray, dtype: int) -> np.ndarray:
    """Round float32 values to `dtype` (nearest-even) and return them as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == DT_F32:
        return a
    if dtype == DT_F16:
        return a.astype(np.float16).astype(np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """Raw storage array (float32 / uint16 bf16 bits / float16) of already-rounded values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == DT_F32:
        return a
    if dtype == DT_F16:
        return a.astype(np.float16)
    return (a.view(np.uint32) >> 16).astype(np.uint16)


class _Builder:
    def __init__(self, name, dtype, seed, in_kind, in_c, in_h, in_w):
        self.name, self.dtype, self.seed = name, dtype, seed
        self.in_kind, self.in_c, self.in_h, self.in_w = in_kind, in_c, in_h, in_w
        self.rng = np.random.default_rng(seed)
        self.layers: List[Layer] = []
        self.groups: List[int] = []
        self.chunks: List[np.ndarray] = []
        self.n_elems = 0
        self.cur_group = 0
        self.flops = 0.0

    # -- blob management: every tensor starts on a 16-element boundary
    def _push(self, arr: np.ndarray) -> int:
        arr = round_to_dtype(arr.reshape(-1), self.dtype)
        off = self.n_elems
        pad = (-arr.size) % 16
        self.chunks.append(arr)
        if pad:
            self.chunks.append(np.zeros(pad, np.float32))
        self.n_elems += arr.size + pad
        return off

    def normal(self, shape, std) -> int:
        return self._push(self.rng.standard_normal(int(np.prod(shape)), dtype=np.float32) * np.float32(std))

    def const(self, n, val) -> int:
        return self._push(np.full(n, val, np.float32))

    def dims(self, idx):
        if idx == -1:
            if self.in_kind == IN_IMAGE:
                return KIND_IMAGE, self.in_c, self.in_h, self.in_w
            if self.in_kind in (IN_SEQ, IN_TOKENS):
                return KIND_SEQ, self.in_c, 1, self.in_w
            return KIND_VEC, self.in_c, 1, 1
        L = self.layers[idx]
        return L.kind, L.c, L.h, L.w

    def add(self, L: Layer) -> int:
        self.layers.append(L)
        self.groups.append(self.cur_group)
        return len(self.layers) - 1

    # -- layer helpers ---------------------------------------------------------
    def conv(self, x, cout, k, stride=1, pad=0, act=ACT_NONE, res=-2, groups=1, std=None,
             bias_std=0.0, w_scale=1.0):
        _, cin, h, w = self.dims(x)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        fan_in = (cin // groups) * k * k
        std = math.sqrt(2.0 / fan_in) if std is None else std
        w_off = self.normal((cout, cin // groups, k, k), std * w_scale)
        b_off = self.normal((cout,), bias_std) if bias_std > 0 else self.const(cout, 0.0)
        self.flops += 2.0 * ho * wo * cout * fan_in
        return self.add(Layer(OP_CONV, x, res, KIND_IMAGE, cout, ho, wo, k, k, stride, pad, groups, act,
                              w_off=w_off, b_off=b_off))

    def linear(self, x, n, act=ACT_NONE, res=-2, std=None, bias_std=0.0):
        kind, c, h, w = self.dims(x)
        if kind == KIND_SEQ:
            k, rows, okind, oh, ow = c, w, KIND_SEQ, 1, w
        else:
            k, rows, okind, oh, ow = c * h * w, 1, KIND_VEC, 1, 1
        std = math.sqrt(2.0 / k) if std is None else std
        w_off = self.normal((n, k), std)
        b_off = self.normal((n,), bias_std) if bias_std > 0 else self.const(n, 0.0)
        self.flops += 2.0 * rows * n * k
        return self.add(Layer(OP_LINEAR, x, res, okind, n, oh, ow, act=act, w_off=w_off, b_off=b_off))

    def maxpool(self, x, k, stride, pad=0):
        _, c, h, w = self.dims(x)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        return self.add(Layer(OP_MAXPOOL, x, -2, KIND_IMAGE, c, ho, wo, k, k, stride, pad))

    def gap(self, x):
        _, c, h, w = self.dims(x)
        return self.add(Layer(OP_GAP, x, -2, KIND_VEC, c, 1, 1))

    def layernorm(self, x, res=-2, eps=1e-12, affine_std=0.0):
        kind, c, h, w = self.dims(x)
        if affine_std > 0:
            g_off = self._push(1.0 + self.rng.standard_normal(c, dtype=np.float32) * np.float32(affine_std))
            be_off = self.normal((c,), affine_std)
        else:
            g_off, be_off = self.const(c, 1.0), self.const(c, 0.0)
        return self.add(Layer(OP_LAYERNORM, x, res, kind, c, h, w, g_off=g_off, be_off=be_off, eps=eps))

    def softmax(self, x):
        kind, c, h, w = self.dims(x)
        return self.add(Layer(OP_SOFTMAX, x, -2, kind, c, h, w))

    def attention(self, x, heads):
        kind, c3, h, w = self.dims(x)
        assert kind == KIND_SEQ and c3 % 3 == 0 and (c3 // 3) % heads == 0
        hd = c3 // 3
        self.flops += 4.0 * w * w * hd
        return self.add(Layer(OP_ATTENTION, x, -2, KIND_SEQ, hd, 1, w, heads=heads))

    def embed(self, hidden, vocab, n_pos, std):
        assert self.in_kind == IN_TOKENS
        tok = self.normal((vocab, hidden), std)
        pos = self.normal((n_pos, hidden), std)
        typ = self.normal((2, hidden), std)
        return self.add(Layer(OP_EMBED, -1, -2, KIND_SEQ, hidden, 1, self.in_w, w_off=tok, g_off=pos,
                              be_off=typ, aux0=vocab, aux1=n_pos))

    def eltwise(self, x, act=ACT_NONE, res=-2, bias_std=0.0):
        kind, c, h, w = self.dims(x)
        b_off = self.normal((c,), bias_std) if bias_std > 0 else -1
        return self.add(Layer(OP_ELTWISE, x, res, kind, c, h, w, act=act, b_off=b_off))

    def concat(self, x, x2):
        kind, c, h, w = self.dims(x)
        kind2, c2, h2, w2 = self.dims(x2)
        assert (kind, h, w) == (kind2, h2, w2)
        return self.add(Layer(OP_CONCAT, x, x2, kind, c + c2, h, w))

    def shuffle(self, x, groups):
        kind, c, h, w = self.dims(x)
        assert c % groups == 0
        return self.add(Layer(OP_SHUFFLE, x, -2, kind, c, h, w, groups=groups))

    def linear_shared(self, x, n, w_off, b_off, act=ACT_NONE, res=-2):
        """A linear layer on a sequence that reuses weights already in the blob (cross-layer sharing)."""
        kind, c, h, w = self.dims(x)
        assert kind == KIND_SEQ
        self.flops += 2.0 * w * n * c
        return self.add(Layer(OP_LINEAR, x, res, KIND_SEQ, n, 1, w, act=act, w_off=w_off, b_off=b_off))

    def next_group(self):
        self.cur_group += 1

    def finish(self) -> Model:
        weights = np.concatenate(self.chunks) if self.chunks else np.zeros(16, np.float32)
        return Model(self.name, self.dtype, self.in_kind, self.in_c, self.in_h, self.in_w, self.layers,
                     weights, list(self.groups), self.cur_group + 1, self.seed, self.flops)


# ---- the networks named by the configurations ----------------------------------
def tiny_cnn(seed=0, dtype=DT_F32, hw=32) -> Model:
    """conv3x3(3->16,s1,p1)+ReLU, conv3x3(16->32,s2,p1)+ReLU, global average pool, FC 32->10."""
    b = _Builder("tiny_cnn", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, 16, 3, 1, 1, ACT_RELU)
    x = b.conv(x, 32, 3, 2, 1, ACT_RELU)
    x = b.gap(x)
    b.linear(x, 10)
    return b.finish()


def resnet(depth=18, seed=1, dtype=DT_BF16, hw=224, n_classes=1000, width=64, res_scale=1.0) -> Model:
    """ResNet-style classifier, v1.5 stride placement, normalisation folded into conv + bias.

    Kernel groups = the four stages (stem and max-pool in the first, pooling and
    classifier in the last)."""
    cfg = {18: ("basic", [2, 2, 2, 2]), 34: ("basic", [3, 4, 6, 3]), 50: ("bottle", [3, 4, 6, 3]),
           101: ("bottle", [3, 4, 23, 3]), 152: ("bottle", [3, 8, 36, 3])}[depth]
    kind, reps = cfg
    b = _Builder(f"resnet{depth}", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, width, 7, 2, 3, ACT_RELU)
    x = b.maxpool(x, 3, 2, 1)
    cin = width
    for stage, n in enumerate(reps):
        if stage:
            b.next_group()
        planes = width << stage
        for i in range(n):
            s = 2 if (stage > 0 and i == 0) else 1
            cout = planes * (4 if kind == "bottle" else 1)
            sc = x
            if s != 1 or cin != cout:
                sc = b.conv(x, cout, 1, s, 0, ACT_NONE)
            if kind == "basic":
                y = b.conv(x, planes, 3, s, 1, ACT_RELU)
                x = b.conv(y, planes, 3, 1, 1, ACT_RELU, res=sc, w_scale=res_scale)
            else:
                y = b.conv(x, planes, 1, 1, 0, ACT_RELU)
                y = b.conv(y, planes, 3, s, 1, ACT_RELU)
                x = b.conv(y, cout, 1, 1, 0, ACT_RELU, res=sc, w_scale=res_scale)
            cin = cout
    x = b.gap(x)
    b.linear(x, n_classes)
    return b.finish()


def vgg16(seed=6, dtype=DT_BF16, hw=224, n_classes=1000, width=64, fc=4096) -> Model:
    """13 conv3x3 + ReLU, 5 max-pool 2x2, flatten (C,H,W), FC-ReLU-FC-ReLU-FC. Groups: 5 conv blocks + FC block."""
    b = _Builder("vgg16", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = -1
    for blk, (mult, n) in enumerate([(1, 2), (2, 2), (4, 3), (8, 3), (8, 3)]):
        if blk:
            b.next_group()
        for _ in range(n):
            x = b.conv(x, width * mult, 3, 1, 1, ACT_RELU)
        x = b.maxpool(x, 2, 2, 0)
    b.next_group()
    x = b.linear(x, fc, ACT_RELU)
    x = b.linear(x, fc, ACT_RELU)
    b.linear(x, n_classes)
    return b.finish()


def mobilenetv2(seed=7, dtype=DT_BF16, hw=224, n_classes=1000) -> Model:
    """MobileNetV2-style: expansion 6, ReLU6 after expand and depthwise, linear projection,
    residual when stride 1 and cin == cout.  Groups: the 7 bottleneck stages."""
    b = _Builder("mobilenetv2", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, 32, 3, 2, 1, ACT_RELU6)
    cin = 32
    table = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    for si, (t, c, n, s) in enumerate(table):
        if si:
            b.next_group()
        for i in range(n):
            stride = s if i == 0 else 1
            inp = x
            y = x
            if t != 1:
                y = b.conv(y, cin * t, 1, 1, 0, ACT_RELU6)
            y = b.conv(y, cin * t, 3, stride, 1, ACT_RELU6, groups=cin * t)
            res = inp if (stride == 1 and cin == c) else -2
            x = b.conv(y, c, 1, 1, 0, ACT_NONE, res=res)
            cin = c
    x = b.conv(x, 1280, 1, 1, 0, ACT_RELU6)
    x = b.gap(x)
    b.linear(x, n_classes)
    return b.finish()


def bert(n_layers=12, hidden=768, heads=12, ffn=3072, seq=128, vocab=30522, seed=4, dtype=DT_F16,
         layers_per_group=3, std=0.02) -> Model:
    """BERT-style post-LN encoder; output = final hidden states [B,S,hidden]."""
    b = _Builder(f"bert_L{n_layers}_H{hidden}", dtype, seed, IN_TOKENS, hidden, 1, seq)
    x = b.embed(hidden, vocab, max(seq, 512), std)
    x = b.layernorm(x)
    for li in range(n_layers):
        if li and li % layers_per_group == 0:
            b.next_group()
        qkv = b.linear(x, 3 * hidden, std=std)
        a = b.attention(qkv, heads)
        o = b.linear(a, hidden, std=std)
        h = b.layernorm(o, res=x)
        f = b.linear(h, ffn, ACT_GELU, std=std)
        f = b.linear(f, hidden, std=std)
        x = b.layernorm(f, res=h)
    return b.finish()


# ---- second workload family: analogues of the paper's remaining models (Sec. IV: albert, densenet201, resnext101,
# ---- shufflenet), same conventions as above (normalisation folded, He-normal weights, zero bias) -----------------
def albert(n_layers=12, hidden=768, heads=12, ffn=3072, seq=128, vocab=30000, embed=128, seed=21, dtype=DT_F16,
           layers_per_group=3, std=0.02) -> Model:
    """ALBERT-style encoder: factorised embedding (vocab x embed, then embed -> hidden) and ONE set of encoder
    weights shared by all layers (every layer's descriptor points at the same offsets of the blob)."""
    b = _Builder(f"albert_L{n_layers}_H{hidden}", dtype, seed, IN_TOKENS, embed, 1, seq)
    x = b.embed(embed, vocab, max(seq, 512), std)
    x = b.layernorm(x)
    x = b.linear(x, hidden, std=std)
    shared = None
    for li in range(n_layers):
        if li and li % layers_per_group == 0:
            b.next_group()
        if shared is None:
            qkv = b.linear(x, 3 * hidden, std=std)
            a = b.attention(qkv, heads)
            o = b.linear(a, hidden, std=std)
            h = b.layernorm(o, res=x)
            f1 = b.linear(h, ffn, ACT_GELU, std=std)
            f2 = b.linear(f1, hidden, std=std)
            x = b.layernorm(f2, res=h)
            shared = [(b.layers[i].w_off, b.layers[i].b_off) for i in (qkv, o, f1, f2)] + \
                     [(b.layers[i].g_off, b.layers[i].be_off) for i in (h, x)]
        else:
            (wq, bq), (wo, bo), (w1, b1), (w2, b2), (g1, e1), (g2, e2) = shared
            qkv = b.linear_shared(x, 3 * hidden, wq, bq)
            a = b.attention(qkv, heads)
            o = b.linear_shared(a, hidden, wo, bo)
            h = b.add(Layer(OP_LAYERNORM, o, x, KIND_SEQ, hidden, 1, seq, g_off=g1, be_off=e1, eps=1e-12))
            f1 = b.linear_shared(h, ffn, w1, b1, ACT_GELU)
            f2 = b.linear_shared(f1, hidden, w2, b2)
            x = b.add(Layer(OP_LAYERNORM, f2, h, KIND_SEQ, hidden, 1, seq, g_off=g2, be_off=e2, eps=1e-12))
    return b.finish()


def densenet(blocks=(6, 12, 24, 16), growth=32, seed=22, dtype=DT_BF16, hw=224, n_classes=1000, bottleneck=4) -> Model:
    """DenseNet-style classifier: every dense layer is conv1x1 (bottleneck x growth) + conv3x3 (growth) whose output
    is concatenated to its input; transitions halve channels (conv1x1) and resolution (2x2 max-pool standing in for
    the average pool).  Kernel groups = the dense blocks."""
    b = _Builder(f"densenet_{'_'.join(map(str, blocks))}", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, 2 * growth, 7, 2, 3, ACT_RELU)
    x = b.maxpool(x, 3, 2, 1)
    c = 2 * growth
    for bi, n in enumerate(blocks):
        if bi:
            b.next_group()
        for _ in range(n):
            y = b.conv(x, bottleneck * growth, 1, 1, 0, ACT_RELU)
            y = b.conv(y, growth, 3, 1, 1, ACT_RELU)
            x = b.concat(x, y)
            c += growth
        if bi + 1 < len(blocks):
            c //= 2
            x = b.conv(x, c, 1, 1, 0, ACT_RELU)
            x = b.maxpool(x, 2, 2, 0)
    x = b.gap(x)
    b.linear(x, n_classes)
    return b.finish()


def resnext(reps=(3, 4, 6, 3), groups=32, width_per_group=4, seed=23, dtype=DT_BF16, hw=224, n_classes=1000,
            res_scale=1.0) -> Model:
    """ResNeXt-style classifier: ResNet bottlenecks whose 3x3 convolution is grouped (`groups` groups of
    `width_per_group` x 2^stage channels).  Kernel groups = the four stages."""
    b = _Builder(f"resnext_{groups}x{width_per_group}d", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, 64, 7, 2, 3, ACT_RELU)
    x = b.maxpool(x, 3, 2, 1)
    cin = 64
    for stage, n in enumerate(reps):
        if stage:
            b.next_group()
        inner = groups * width_per_group << stage
        cout = 256 << stage
        for i in range(n):
            s = 2 if (stage > 0 and i == 0) else 1
            sc = x
            if s != 1 or cin != cout:
                sc = b.conv(x, cout, 1, s, 0, ACT_NONE)
            y = b.conv(x, inner, 1, 1, 0, ACT_RELU)
            y = b.conv(y, inner, 3, s, 1, ACT_RELU, groups=groups)
            x = b.conv(y, cout, 1, 1, 0, ACT_RELU, res=sc, w_scale=res_scale)
            cin = cout
    x = b.gap(x)
    b.linear(x, n_classes)
    return b.finish()


def shufflenet(groups=8, reps=(4, 8, 4), base=384, seed=24, dtype=DT_BF16, hw=224, n_classes=1000, res_scale=0.5) -> Model:
    """ShuffleNet-style classifier (v1 units): grouped 1x1 -> channel shuffle -> depthwise 3x3 -> grouped 1x1,
    added to the input (stride 1) or to a strided 1x1 projection of it (stride 2, standing in for the pooled
    concatenation); the last convolution of every unit is scaled by `res_scale` to keep the un-normalised residual
    stream bounded.  Channel counts are multiples of 8 x groups.  Kernel groups = the three stages."""
    b = _Builder(f"shufflenet_g{groups}", dtype, seed, IN_IMAGE, 3, hw, hw)
    x = b.conv(-1, 24, 3, 2, 1, ACT_RELU)
    x = b.maxpool(x, 3, 2, 1)
    cin = 24
    for stage, n in enumerate(reps):
        if stage:
            b.next_group()
        cout = base << stage
        mid = cout // 4
        for i in range(n):
            s = 2 if i == 0 else 1
            g1 = 1 if cin % groups else groups          # the 24-channel stem output is not divisible: dense 1x1 there
            sc = x if (s == 1 and cin == cout) else b.conv(x, cout, 1, s, 0, ACT_NONE)
            y = b.conv(x, mid, 1, 1, 0, ACT_RELU, groups=g1)
            y = b.shuffle(y, groups)
            y = b.conv(y, mid, 3, s, 1, ACT_NONE, groups=mid)
            x = b.conv(y, cout, 1, 1, 0, ACT_RELU, res=sc, groups=groups, w_scale=res_scale)
            cin = cout
    x = b.gap(x)
    b.linear(x, n_classes)
    return b.finish()


def single_layer(op: str, dtype=DT_BF16, seed=0, **kw) -> Model:
    """A one- or two-layer model used to test each kernel through the same entry points."""
    if op == "conv":
        b = _Builder("conv", dtype, seed, IN_IMAGE, kw["cin"], kw["h"], kw["w"])
        res = -2
        x = -1
        if kw.get("residual"):
            # the residual operand must have the output's shape: produce it with a first conv
            res = b.conv(-1, kw["cout"], kw["k"], kw.get("stride", 1), kw.get("pad", 0), groups=kw.get("groups", 1),
                         bias_std=kw.get("bias_std", 0.0))
        b.conv(x, kw["cout"], kw["k"], kw.get("stride", 1), kw.get("pad", 0), kw.get("act", ACT_NONE), res=res,
               groups=kw.get("groups", 1), bias_std=kw.get("bias_std", 0.0))
    elif op == "linear":
        b = _Builder("linear", dtype, seed, IN_SEQ, kw["k"], 1, kw["rows"])
        res = -1 if kw.get("residual") else -2
        b.linear(-1, kw["n"], kw.get("act", ACT_NONE), res=res, std=kw.get("std"), bias_std=kw.get("bias_std", 0.0))
    elif op == "maxpool":
        b = _Builder("maxpool", dtype, seed, IN_IMAGE, kw["c"], kw["h"], kw["w"])
        b.maxpool(-1, kw["k"], kw["stride"], kw.get("pad", 0))
    elif op == "gap":
        b = _Builder("gap", dtype, seed, IN_IMAGE, kw["c"], kw["h"], kw["w"])
        b.gap(-1)
    elif op == "stem":
        # first convolution of an image model (few input channels) followed by a second convolution
        b = _Builder("stem", dtype, seed, IN_IMAGE, kw["cin"], kw["h"], kw["w"])
        x = b.conv(-1, kw["cout"], kw["k"], kw.get("stride", 1), kw.get("pad", 0), kw.get("act", ACT_RELU), bias_std=kw.get("bias_std", 0.0))
        b.conv(x, kw.get("cout2", kw["cout"]), 1, 1, 0, ACT_NONE)
    elif op == "gapfc":
        # global average pool + classifier (+ an optional second linear layer, so that the classifier is not the last layer)
        b = _Builder("gapfc", dtype, seed, IN_IMAGE, kw["c"], kw["h"], kw["w"])
        x = b.gap(-1)
        x = b.linear(x, kw["n"], kw.get("act", ACT_NONE), std=kw.get("std"), bias_std=kw.get("bias_std", 0.0))
        if kw.get("then"):
            b.linear(x, kw["then"], std=kw.get("std"))
    elif op == "layernorm":
        b = _Builder("layernorm", dtype, seed, IN_SEQ, kw["width"], 1, kw["rows"])
        res = -2
        if kw.get("residual"):
            res = b.eltwise(-1, ACT_NONE, bias_std=1.0)
        b.layernorm(-1, res=res, eps=kw.get("eps", 1e-12), affine_std=kw.get("affine_std", 0.0))
    elif op == "softmax":
        b = _Builder("softmax", dtype, seed, IN_SEQ, kw["width"], 1, kw["rows"])
        b.softmax(-1)
    elif op == "attention":
        b = _Builder("attention", dtype, seed, IN_SEQ, 3 * kw["hidden"], 1, kw["seq"])
        b.attention(-1, kw["heads"])
    elif op == "embed":
        b = _Builder("embed", dtype, seed, IN_TOKENS, kw["hidden"], 1, kw["seq"])
        b.embed(kw["hidden"], kw["vocab"], kw.get("n_pos", kw["seq"]), kw.get("std", 0.02))
    elif op == "eltwise":
        b = _Builder("eltwise", dtype, seed, IN_SEQ, kw["width"], 1, kw["rows"])
        res = -1 if kw.get("residual") else -2
        b.eltwise(-1, kw.get("act", ACT_NONE), res=res, bias_std=kw.get("bias_std", 0.0))
    elif op == "concat":
        # a sequence input concatenated with an element-wise copy of itself plus a bias (two distinct operands)
        b = _Builder("concat", dtype, seed, IN_SEQ, kw["c0"], 1, kw["rows"])
        if kw["c1"] == kw["c0"]:
            other = b.eltwise(-1, ACT_NONE, bias_std=1.0)
        else:
            other = b.linear(-1, kw["c1"], std=0.1, bias_std=0.5)
        b.concat(-1, other)
    elif op == "shuffle":
        b = _Builder("shuffle", dtype, seed, IN_IMAGE, kw["c"], kw["h"], kw["w"])
        b.shuffle(-1, kw["groups"])
    else:
        raise ValueError(op)
    return b.finish()


# ---- inputs -------------------------------------------------------------------
def make_input(m: Model, batch: int, seed: Optional[int] = None, dist: str = "normal") -> np.ndarray:
    """Seeded input in logical layout: float32 values already rounded to the model dtype, or int32 token ids."""
    rng = np.random.default_rng(10_000 + (m.seed if seed is None else seed))
    shape = m.in_shape(batch)
    if m.in_kind == IN_TOKENS:
        vocab = m.layers[0].aux0
        return rng.integers(0, vocab, size=shape, dtype=np.int32)
    if dist == "uniform":
        x = rng.random(shape, dtype=np.float32)
    else:
        x = rng.standard_normal(shape, dtype=np.float32)
    return round_to_dtype(x, m.dtype)


def poisson_arrivals(rate_per_s: float, duration_s: float, model_index: int) -> np.ndarray:
    """Open-loop arrival times (seconds) with exponential gaps, generated up front."""
    rng = np.random.default_rng(1000 + model_index)
    n = int(rate_per_s * duration_s * 1.5) + 16
    t = np.cumsum(rng.exponential(1.0 / rate_per_s, size=n))
    return t[t < duration_s]


# ---- the five configurations ----------------------------------------------------
def config_models(cfg: int, small: bool = False) -> List[Model]:
    """Models of configuration `cfg` (0-based index into the configuration list).

    `small=True` shrinks spatial size / depth so that a CPU check finishes in seconds
    while keeping every layer type and several tiles per kernel."""
    if cfg == 0:
        return [tiny_cnn(seed=0)]
    if cfg == 1:
        hw = 64 if small else 224
        return [resnet(18, seed=1, hw=hw), resnet(18, seed=2, hw=hw)]
    if cfg == 2:
        if small:
            return [resnet(50, seed=3, hw=64), bert(2, 128, 4, 512, 48, vocab=1000, seed=4)]
        return [resnet(50, seed=3), bert(seed=4)]
    if cfg == 3:
        if small:
            return [resnet(50, seed=5, hw=64), vgg16(seed=6, hw=32, width=16, fc=256), mobilenetv2(seed=7, hw=64, dtype=DT_F16),
                    bert(2, 128, 4, 512, 48, vocab=1000, seed=8)]
        return [resnet(50, seed=5), vgg16(seed=6), mobilenetv2(seed=7, dtype=DT_F16), bert(seed=8)]
    if cfg == 4:
        if small:
            return [bert(2, 128, 4, 512, 48, vocab=1000, seed=9 + i, dtype=DT_BF16) for i in range(3)] + \
                   [resnet(152, seed=12, hw=64, res_scale=0.25)]
        return [bert(24, 1024, 16, 4096, 384, seed=9 + i, dtype=DT_BF16) for i in range(3)] + \
               [resnet(152, seed=12, res_scale=0.25)]
    # second workload family: analogues of two of the paper's mixes (Sec. IV: Mix 2 = albert + densenet201,
    # Mix 5 = resnext101 + shufflenet), at the public depths of the smaller members of each family
    if cfg == 5:
        if small:
            return [albert(2, 128, 4, 512, 48, vocab=1000, embed=64, seed=21), densenet((2, 4, 2), 16, seed=22, hw=64)]
        return [albert(seed=21), densenet(seed=22)]
    if cfg == 6:
        if small:
            return [resnext((2, 1, 1), 8, 4, seed=23, hw=64, res_scale=0.5), shufflenet(4, (2, 2), 128, seed=24, hw=64)]
        return [resnext(seed=23, res_scale=0.5), shufflenet(seed=24)]
    # a two-worker mix of large-batch models whose kernel groups need very different CU counts: VGG-16's convolution
    # blocks scale with the CUs they get while its fully connected block streams 250 MB of weights and saturates the
    # memory system on a fraction of them; BERT-large is matrix-core-bound throughout (the paper's "feasible combinations"
    # of a high- and a low-CU-need model, Sec. IV-A)
    if cfg == 7:
        if small:
            return [vgg16(seed=31, hw=32, width=16, fc=256), bert(2, 128, 4, 512, 48, vocab=1000, seed=32, dtype=DT_BF16)]
        return [vgg16(seed=31), bert(24, 1024, 16, 4096, 384, seed=32, dtype=DT_BF16)]
    raise ValueError(cfg)
