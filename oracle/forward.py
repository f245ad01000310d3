"""Python driver of the C forward-pass oracle -- TEST INFRASTRUCTURE ONLY.

Walks a layer table (records with fields op, c_in, c_out, k, stride, pad, groups,
act, in_from, res_from) and applies the plain per-layer definitions of
`forward.c` to NCHW float32 tensors.

Precision modes
  "fp32": weights/inputs as given; every output element is a double sum rounded
          once to float.
  "bf16": weights and the input are rounded to bfloat16 (nearest-even) once; every
          layer's output (after bias, residual and activation) is rounded to
          bfloat16 before the next layer reads it; biases stay float32; the last
          layer's output (the logits) stays float32.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import build

OP_CONV, OP_MAXPOOL, OP_GAVGPOOL, OP_FC = 0, 1, 2, 3

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        fp, dp = C.POINTER(C.c_float), C.POINTER(C.c_double)
        _lib.orc_conv2d.argtypes = [fp, C.c_int, C.c_int, C.c_int, fp, fp, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_int, fp, C.c_int, C.c_int, fp]
        _lib.orc_maxpool2d.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, fp]
        _lib.orc_gavgpool.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_int, fp]
        _lib.orc_fc.argtypes = [fp, C.c_int, fp, fp, C.c_int, C.c_int, C.c_int, fp]
        _lib.orc_bf16_round.argtypes = [fp, C.c_int64]
        _lib.orc_bf16_round_scalar.argtypes = [C.c_float]
        _lib.orc_bf16_round_scalar.restype = C.c_float
        _lib.orc_batchnorm.argtypes = [dp, C.c_int, C.c_int, dp, dp, dp, dp, C.c_double, dp]
        for f in ("orc_conv2d", "orc_maxpool2d", "orc_gavgpool", "orc_fc", "orc_bf16_round", "orc_batchnorm"):
            getattr(_lib, f).restype = None
    return _lib


def _fp(a):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_float))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def bf16_round(a):
    """Round a float32 array to bfloat16 (nearest, ties to even), returned as float32."""
    out = _f32(a).copy()
    lib().orc_bf16_round(_fp(out), out.size)
    return out


def conv2d(x, w, b=None, stride=1, pad=0, groups=1, res=None, act=0, round_bf16=False):
    x, w = _f32(x), _f32(w)
    c, h, wd = x.shape
    cout, cg, k, k2 = w.shape
    assert k == k2 and cg * groups == c and cout % groups == 0
    ho, wo = (h + 2 * pad - k) // stride + 1, (wd + 2 * pad - k) // stride + 1
    y = np.empty((cout, ho, wo), np.float32)
    b = None if b is None else _f32(b)
    res = None if res is None else _f32(res)
    if res is not None:
        assert res.shape == y.shape
    lib().orc_conv2d(_fp(x), c, h, wd, _fp(w), _fp(b), cout, k, stride, pad, groups, _fp(res), act,
                     int(round_bf16), _fp(y))
    return y


def maxpool2d(x, k, stride, pad=0):
    x = _f32(x)
    c, h, w = x.shape
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    y = np.empty((c, ho, wo), np.float32)
    lib().orc_maxpool2d(_fp(x), c, h, w, k, stride, pad, _fp(y))
    return y


def gavgpool(x, round_bf16=False):
    x = _f32(x)
    c, h, w = x.shape
    y = np.empty((c, 1, 1), np.float32)
    lib().orc_gavgpool(_fp(x), c, h, w, int(round_bf16), _fp(y))
    return y


def fc(x, w, b=None, act=0, round_bf16=False):
    x, w = _f32(x).reshape(-1), _f32(w)
    n, k = w.shape
    assert k == x.size
    y = np.empty((n,), np.float32)
    b = None if b is None else _f32(b)
    lib().orc_fc(_fp(x), k, _fp(w), _fp(b), n, act, int(round_bf16), _fp(y))
    return y


def batchnorm(x, gamma, beta, mean, var, eps):
    x = np.ascontiguousarray(x, np.float64)
    c = x.shape[0]
    y = np.empty_like(x)
    dp = lambda a: np.ascontiguousarray(a, np.float64).ctypes.data_as(C.POINTER(C.c_double))
    lib().orc_batchnorm(dp(x), c, x.size // c, dp(gamma), dp(beta), dp(mean), dp(var), float(eps),
                        y.ctypes.data_as(C.POINTER(C.c_double)))
    return y


def forward(layers, weights, x, dtype="fp32", return_all=False):
    """Logits (float32 vector) of one input `x` (C, H, W); `weights[l]` = (w, b) or (None, None)."""
    bf = dtype == "bf16"
    x = _f32(x)
    if bf:
        x = bf16_round(x)
    outs = []
    n = len(layers)
    for l, L in enumerate(layers):
        src = x if L.in_from < 0 else outs[L.in_from]
        rnd = bf and l != n - 1
        w, b = weights[l]
        if bf and w is not None:
            w = bf16_round(w)
        if L.op == OP_CONV:
            res = outs[L.res_from] if L.res_from >= 0 else None
            y = conv2d(src, w, b, L.stride, L.pad, L.groups, res, L.act, rnd)
        elif L.op == OP_MAXPOOL:
            y = maxpool2d(src, L.k, L.stride, L.pad)
        elif L.op == OP_GAVGPOOL:
            y = gavgpool(src, rnd)
        elif L.op == OP_FC:
            y = fc(src, w, b, L.act, rnd).reshape(-1, 1, 1)
        else:
            raise ValueError(L.op)
        outs.append(y)
    logits = outs[-1].reshape(-1)
    return (logits, outs) if return_all else logits
