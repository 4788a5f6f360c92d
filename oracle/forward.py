"""Forward-pass oracle: interprets a layer graph with the plain-C routines of fwd_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the CPU-baseline
leg of the benchmark; never by the product path.  Shares no code with the GPU
library (the only common input is the `workloads` description of each network).

The paper runs stock inference models (Sec. IV-A) and gives no network
mathematics; the layer semantics are the textbook ones listed in
`workloads/graphs.py`.  Activations are fp64 throughout, in logical layouts
([B,C,H,W] images, [B,S,Hd] sequences, [B,n] vectors).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fwd_oracle.c")
_LIB = os.path.join(_HERE, "libfwd_oracle.so")

# operator / tensor-kind codes of the layer descriptor (values fixed by the descriptor format)
OP_CONV, OP_LINEAR, OP_MAXPOOL, OP_GAP, OP_LAYERNORM, OP_SOFTMAX, OP_ATTENTION, OP_EMBED, OP_ELTWISE, OP_CONCAT, OP_SHUFFLE = \
    range(1, 12)
KIND_IMAGE, KIND_SEQ, KIND_VEC = range(3)
IN_IMAGE, IN_TOKENS, IN_SEQ, IN_VEC = range(4)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over output channels / rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


I64 = ctypes.c_int64


# ---- operator wrappers (each a thin call of the C definition) ---------------------
def conv2d(x, w, b, stride=1, pad=0, groups=1):
    x = _f64(x); w = _f32(w); b = _f32(b)
    n, c, h, wd = x.shape
    cout, cig, kh, kw = w.shape
    assert cig * groups == c and cout % groups == 0
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.empty((n, cout, ho, wo), np.float64)
    lib().orc_conv2d(_d(x), n, c, h, wd, _f(w), _f(b), cout, kh, kw, stride, pad, groups, _d(y))
    return y


def linear(x, w, b):
    x = _f64(x); w = _f32(w); b = _f32(b)
    m, k = x.shape
    n = w.shape[0]
    assert w.shape[1] == k
    y = np.empty((m, n), np.float64)
    lib().orc_linear(_d(x), I64(m), I64(k), _f(w), _f(b), I64(n), _d(y))
    return y


def maxpool(x, k, stride, pad=0):
    x = _f64(x)
    n, c, h, w = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, ho, wo), np.float64)
    lib().orc_maxpool(_d(x), n, c, h, w, k, k, stride, pad, _d(y))
    return y


def gap(x):
    x = _f64(x)
    n, c, h, w = x.shape
    y = np.empty((n, c), np.float64)
    lib().orc_gap(_d(x), n, c, h * w, _d(y))
    return y


def layernorm(x, gamma, beta, eps):
    x = _f64(x); gamma = _f32(gamma); beta = _f32(beta)
    width = x.shape[-1]
    rows = x.size // width
    y = np.empty_like(x)
    lib().orc_layernorm(_d(x), I64(rows), I64(width), _f(gamma), _f(beta), ctypes.c_double(eps), _d(y))
    return y


def softmax(x):
    x = _f64(x)
    width = x.shape[-1]
    y = np.empty_like(x)
    lib().orc_softmax(_d(x), I64(x.size // width), I64(width), _d(y))
    return y


def attention(qkv, heads):
    qkv = _f64(qkv)
    b, s, h3 = qkv.shape
    hd = h3 // 3
    out = np.empty((b, s, hd), np.float64)
    scratch = np.empty(b * heads * s, np.float64)
    lib().orc_attention(_d(qkv), b, s, hd, heads, _d(out), _d(scratch))
    return out


def embed(ids, tok, pos, typ):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    tok = _f32(tok); pos = _f32(pos); typ = _f32(typ)
    b, s = ids.shape
    hd = tok.shape[1]
    assert ids.min() >= 0 and ids.max() < tok.shape[0] and s <= pos.shape[0]
    y = np.empty((b, s, hd), np.float64)
    lib().orc_embed(ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), b, s, hd, _f(tok), _f(pos), _f(typ), _d(y))
    return y


def eltwise(x, bias, res, act, channel_axis):
    """y = act(x + bias[channel] + res)."""
    x = _f64(x); bias = _f32(bias)
    res = None if res is None else _f64(res)
    channels = x.shape[channel_axis]
    inner = int(np.prod(x.shape[channel_axis + 1:])) if channel_axis + 1 < x.ndim else 1
    y = np.empty_like(x)
    lib().orc_eltwise(_d(x), _f(bias), None if res is None else _d(res), _d(y), I64(x.size), I64(channels),
                      I64(inner), act)
    return y


# ---- graph interpreter ---------------------------------------------------------------
def _round_storage(y: np.ndarray, dtype: int) -> np.ndarray:
    """Round to bf16 (dtype 1) or fp16 (dtype 2), nearest-even, and return as fp64."""
    a = np.ascontiguousarray(y, dtype=np.float32)
    if dtype == 2:
        return a.astype(np.float16).astype(np.float64)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape).astype(np.float64)


def run_model(model, x_in: np.ndarray, keep_all: bool = False, storage_dtype: int = 0):
    """Forward pass of `model` (a workloads.Model) on a logical-layout input batch.

    Returns the last layer's output as fp64 (or the list of every layer's output).

    `storage_dtype` = 1 (bf16) or 2 (fp16) additionally rounds every layer's output except the last
    to that type, i.e. it models a path that stores activations in 16 bits between layers while doing
    all arithmetic exactly.  It separates storage rounding from arithmetic error; the default (0)
    is the plain definition."""
    W = model.weights
    outs: List[Optional[np.ndarray]] = []

    def src(i):
        return x_in if i == -1 else outs[i]

    def dims_of(i):
        if i == -1:
            return model.in_c, model.in_h, model.in_w
        L = model.layers[i]
        return L.c, L.h, L.w

    for L in model.layers:
        x = src(L.in0)
        res = None if L.in1 == -2 else src(L.in1)
        if L.op == OP_CONV:
            cin, _, _ = dims_of(L.in0)
            cig = cin // L.groups
            w = W[L.w_off:L.w_off + L.c * cig * L.kh * L.kw].reshape(L.c, cig, L.kh, L.kw)
            y = conv2d(x, w, None, L.stride, L.pad, L.groups)
            bias = W[L.b_off:L.b_off + L.c] if L.b_off >= 0 else None
            y = eltwise(y, bias, res, L.act, 1)
        elif L.op == OP_LINEAR:
            b = x.shape[0]
            if L.kind == KIND_SEQ:
                k = x.shape[-1]
                x2 = _f64(x).reshape(-1, k)
            else:
                x2 = _f64(x).reshape(b, -1)       # images flatten in (C,H,W) order
                k = x2.shape[1]
            w = W[L.w_off:L.w_off + L.c * k].reshape(L.c, k)
            y = linear(x2, w, None)
            y = y.reshape(b, -1, L.c) if L.kind == KIND_SEQ else y
            bias = W[L.b_off:L.b_off + L.c] if L.b_off >= 0 else None
            y = eltwise(y, bias, res, L.act, y.ndim - 1)
        elif L.op == OP_MAXPOOL:
            y = maxpool(x, L.kh, L.stride, L.pad)
        elif L.op == OP_GAP:
            y = gap(x)
        elif L.op == OP_LAYERNORM:
            xs = _f64(x) if res is None else _f64(x) + _f64(res)
            y = layernorm(xs, W[L.g_off:L.g_off + L.c], W[L.be_off:L.be_off + L.c], L.eps)
        elif L.op == OP_SOFTMAX:
            y = softmax(x)
        elif L.op == OP_ATTENTION:
            y = attention(x, L.heads)
        elif L.op == OP_EMBED:
            hd = L.c
            tok = W[L.w_off:L.w_off + L.aux0 * hd].reshape(L.aux0, hd)
            pos = W[L.g_off:L.g_off + L.aux1 * hd].reshape(L.aux1, hd)
            typ = W[L.be_off:L.be_off + 2 * hd].reshape(2, hd)
            y = embed(x, tok, pos, typ)
        elif L.op == OP_ELTWISE:
            bias = W[L.b_off:L.b_off + L.c] if L.b_off >= 0 else None
            y = eltwise(x, bias, res, L.act, 1 if L.kind == KIND_IMAGE else np.ndim(x) - 1)
        elif L.op == OP_CONCAT:
            # channels are axis 1 of an image [B,C,H,W] and the last axis of a sequence / vector
            y = np.concatenate([_f64(x), _f64(res)], axis=1 if L.kind == KIND_IMAGE else -1)
        elif L.op == OP_SHUFFLE:
            # channel shuffle: view the C channels as (groups, C/groups), transpose, flatten
            ax = 1 if L.kind == KIND_IMAGE else np.ndim(x) - 1
            xs = np.moveaxis(_f64(x), ax, -1)
            n = L.c // L.groups
            ys = xs.reshape(xs.shape[:-1] + (L.groups, n)).swapaxes(-1, -2).reshape(xs.shape)
            y = np.moveaxis(ys, -1, ax)
        else:
            raise ValueError(f"unknown op {L.op}")
        if storage_dtype and L is not model.layers[-1]:
            y = _round_storage(y, storage_dtype)
        outs.append(y)
        if not keep_all:
            # free tensors no later layer reads
            idx = len(outs) - 1
            for j in range(idx):
                if outs[j] is not None and not any(
                        (M.in0 == j or M.in1 == j) for M in model.layers[idx + 1:]):
                    outs[j] = None
    return outs if keep_all else outs[-1]
