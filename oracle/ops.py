"""Operator definitions for the oracle (test infrastructure, see package doc).

The paper runs unchanged framework operators (Section 5, "Experimental
Setup"): what a task computes is the standard inference-time definition of
each layer. Every function takes/returns fp32 NCHW arrays and does its
arithmetic in fp64. No blocking, no fusion: one formula per function.
"""
from __future__ import annotations

import numpy as np


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def _out(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def out_size(size: int, k: int, stride: int, pad: int) -> int:
    """Number of window positions along one axis."""
    return (size + 2 * pad - k) // stride + 1


def conv2d(x, w, stride: int, pad: int):
    """Dense cross-correlation: y[n,o,i,j] = sum_{c,a,b} w[o,c,a,b] * xp[n,c,i*s+a,j*s+b],
    xp = x zero-padded by ``pad`` on each spatial side."""
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    o, c2, k, k2 = w.shape
    assert c == c2 and k == k2
    ho, wo = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((n, o, ho, wo))
    for a in range(k):
        for b in range(k):
            tap = xp[:, :, a:a + stride * (ho - 1) + 1:stride, b:b + stride * (wo - 1) + 1:stride]
            # contraction over input channels for this tap (a matmul per image)
            y += np.matmul(w[:, :, a, b][None], tap.reshape(n, c, ho * wo)).reshape(n, o, ho, wo)
    return _out(y)


def conv1x1(x, w):
    """Pointwise convolution: y[n,o,i,j] = sum_c w[o,c] * x[n,c,i,j]."""
    w = _f64(w)
    return conv2d(x, w[:, :, None, None], 1, 0)


def conv3x3(x, w, stride: int, pad: int):
    return conv2d(x, w, stride, pad)


def dwconv(x, w, stride: int):
    """Depthwise k x k, pad k//2: y[n,c,i,j] = sum_{a,b} w[c,a,b] * xp[n,c,i*s+a,j*s+b]."""
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    c2, k, k2 = w.shape
    assert c == c2 and k == k2
    pad = k // 2
    ho, wo = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    y = np.zeros((n, c, ho, wo))
    for a in range(k):
        for b in range(k):
            tap = xp[:, :, a:a + stride * (ho - 1) + 1:stride, b:b + stride * (wo - 1) + 1:stride]
            y += w[None, :, a, b, None, None] * tap
    return _out(y)


def bn_act(x, gamma, beta, mean, var, eps: float, relu: bool):
    """Inference batch norm: y = gamma * (x - mean) / sqrt(var + eps) + beta, then optional max(.,0)."""
    x = _f64(x)
    g, b, m, v = (_f64(t)[None, :, None, None] for t in (gamma, beta, mean, var))
    y = g * (x - m) / np.sqrt(v + eps) + b
    if relu:
        y = np.maximum(y, 0.0)
    return _out(y)


def relu(x):
    return _out(np.maximum(_f64(x), 0.0))


def add_n(xs):
    """Elementwise sum, accumulated left to right."""
    y = _f64(xs[0]).copy()
    for t in xs[1:]:
        assert t.shape == xs[0].shape
        y += _f64(t)
    return _out(y)


def concat(xs, lo, hi):
    """Stack channel slices xs[j][:, lo[j]:hi[j]] along C, in order."""
    return _out(np.concatenate([_f64(t)[:, l:h] for t, l, h in zip(xs, lo, hi)], axis=1))


def pool3x3(x, mode: str, stride: int, pad: int):
    """3x3 window. 'max': maximum over in-bounds taps. 'avg': sum of in-bounds taps
    divided by their count (padding is excluded from the divisor)."""
    x = _f64(x)
    n, c, h, w = x.shape
    ho, wo = out_size(h, 3, stride, pad), out_size(w, 3, stride, pad)
    fill = -np.inf if mode == "max" else 0.0
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)), constant_values=fill)
    ones = np.pad(np.ones((1, 1, h, w)), ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    acc = np.full((n, c, ho, wo), fill)
    cnt = np.zeros((1, 1, ho, wo))
    for a in range(3):
        for b in range(3):
            sl = (slice(None), slice(None),
                  slice(a, a + stride * (ho - 1) + 1, stride), slice(b, b + stride * (wo - 1) + 1, stride))
            if mode == "max":
                acc = np.maximum(acc, xp[sl])
            else:
                acc = acc + xp[sl]
                cnt = cnt + ones[sl]
    return _out(acc if mode == "max" else acc / cnt)


def global_avgpool(x):
    return _out(_f64(x).mean(axis=(2, 3), keepdims=True))


def fc(x, w, b):
    """y[n,o] = sum_c w[o,c] * x[n,c] + b[o], on [n,c,1,1] tensors."""
    x, w, b = _f64(x), _f64(w), _f64(b)
    n, c, h, wd = x.shape
    assert h == 1 and wd == 1
    return _out((x.reshape(n, c) @ w.T + b[None]).reshape(n, -1, 1, 1))
