"""Seeded random weights, biases and inputs for the layer tables in `nets`.

Recipe (stated again in the design notes):
  * one numpy `Generator(PCG64)` child stream per (task seed, layer, tensor) via
    `SeedSequence`, so a tensor does not depend on generation order;
  * conv / FC weights: He-normal, std = sqrt(2 / fan_in), fan_in = (c_in/groups)*k*k
    (FC: c_in), drawn in float64;
  * layers flagged `has_bn`: gamma ~ U(0.5, 1.5), beta ~ N(0, 0.1^2), mean ~ N(0, 0.1^2),
    var ~ U(0.5, 1.5), eps = 1e-5, folded into (w, b) in float64 by `fold_bn`;
  * other conv / FC layers: bias ~ N(0, 0.05^2);
  * the folded tensors are cast to float32 once; those float32 arrays are THE
    weights handed, identically, to every consumer;
  * inputs: float32, U(0,1) ("uniform") or N(0,1) ("normal").
"""
from __future__ import annotations

import numpy as np

from .nets import OP_CONV, OP_FC

BN_EPS = 1e-5


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *key])))


def fold_bn(w, gamma, beta, mean, var, eps=BN_EPS):
    """Return (w', b') with w'[o] = w[o]*gamma[o]/sqrt(var[o]+eps), b'[o] = beta[o]-mean[o]*gamma[o]/sqrt(var[o]+eps).

    Pure data preparation in float64; a test checks it against an unfused
    convolution followed by batch normalisation.
    """
    w = np.asarray(w, dtype=np.float64)
    scale = np.asarray(gamma, np.float64) / np.sqrt(np.asarray(var, np.float64) + eps)
    wf = w * scale.reshape((-1,) + (1,) * (w.ndim - 1))
    bf = np.asarray(beta, np.float64) - np.asarray(mean, np.float64) * scale
    return wf, bf


def make_bn(seed: int, layer_index: int, c: int):
    g = _rng(seed, layer_index, 1)
    gamma = g.uniform(0.5, 1.5, c)
    beta = g.normal(0.0, 0.1, c)
    mean = g.normal(0.0, 0.1, c)
    var = g.uniform(0.5, 1.5, c)
    return gamma, beta, mean, var


def make_raw_conv(seed: int, layer_index: int, L):
    """Unfolded float64 conv weight of layer L (before any BN fold)."""
    cg = L.c_in // L.groups
    fan_in = cg * L.k * L.k
    return _rng(seed, layer_index, 0).normal(0.0, np.sqrt(2.0 / fan_in), (L.c_out, cg, L.k, L.k))


def make_weights(layers, seed: int):
    """Per layer: (w float32, b float32) for conv/FC layers, (None, None) otherwise."""
    out = []
    for i, L in enumerate(layers):
        if L.op == OP_CONV:
            w = make_raw_conv(seed, i, L)
            if L.has_bn:
                w, b = fold_bn(w, *make_bn(seed, i, L.c_out))
            else:
                b = _rng(seed, i, 2).normal(0.0, 0.05, L.c_out)
            out.append((np.ascontiguousarray(w, dtype=np.float32), np.ascontiguousarray(b, dtype=np.float32)))
        elif L.op == OP_FC:
            w = _rng(seed, i, 0).normal(0.0, np.sqrt(2.0 / L.c_in), (L.c_out, L.c_in))
            b = _rng(seed, i, 2).normal(0.0, 0.05, L.c_out)
            out.append((np.ascontiguousarray(w, dtype=np.float32), np.ascontiguousarray(b, dtype=np.float32)))
        else:
            out.append((None, None))
    return out


def make_inputs(in_shape, seed: int, count: int, dist: str):
    """`count` float32 inputs of shape (C, H, W), stacked as (count, C, H, W)."""
    g = _rng(seed, 1 << 20)
    shape = (count,) + tuple(in_shape)
    x = g.uniform(0.0, 1.0, shape) if dist == "uniform" else g.normal(0.0, 1.0, shape)
    return np.ascontiguousarray(x, dtype=np.float32)
