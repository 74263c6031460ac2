"""Gradients of a DAG for the oracle (test infrastructure, see package doc).

Section 5 of the paper ("Training", the batch-32 training throughput figure)
replays a whole training iteration - forward pass, backward pass and weight
update - as one recorded schedule; what is computed is the framework's ordinary
backward pass. This module states that computation once, plainly: for the scalar

    L = sum over output nodes o of  <value[o], seed[o]>

it returns dL/d(value[v]) for every node and dL/d(weight) for every weight
tensor, each operator by the textbook vector-Jacobian product of the formula
in module ``ops``, nodes visited in descending id, fp64 arithmetic throughout.

Readings (the paper does not go below "the framework's backward pass"):
* batch norm keeps its statistics fixed (the inference-form affine map of
  ``ops.bn_act``), so gamma and beta get gradients, mean and var do not;
* a max pool sends the gradient to the first tap, in row-major window order,
  that attains the maximum; an average pool divides by the number of in-bounds
  taps, as the forward pass does;
* activations that the backward pass reads are the forward pass's stored values.

Parity status: pinned against central finite differences of an fp64 forward
pass on tiny DAGs and against torch.autograd (CPU, fp64) operator by operator.
No HIP counterpart exists yet: nothing on the GPU is compared with this module.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np

from .forward import eval_node


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def _taps(k, stride, ho, wo):
    for a in range(k):
        for b in range(k):
            yield a, b, (slice(None), slice(None),
                         slice(a, a + stride * (ho - 1) + 1, stride), slice(b, b + stride * (wo - 1) + 1, stride))


def _unpad(xp, pad):
    return xp[:, :, pad:xp.shape[2] - pad, pad:xp.shape[3] - pad] if pad else xp


def conv2d_vjp(x, w, stride, pad, dy):
    """y[n,o,i,j] = sum w[o,c,a,b] xp[n,c,i s+a,j s+b]  =>
    dxp[n,c,i s+a,j s+b] += sum_o w[o,c,a,b] dy[n,o,i,j];  dw[o,c,a,b] = sum_{n,i,j} dy[n,o,i,j] xp[n,c,i s+a,j s+b]."""
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    n, c, h, wd = x.shape
    o, _, k, _ = w.shape
    ho, wo = dy.shape[2], dy.shape[3]
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    dyf = dy.reshape(n, o, ho * wo)
    for a, b, sl in _taps(k, stride, ho, wo):
        dxp[sl] += np.matmul(w[:, :, a, b].T[None], dyf).reshape(n, c, ho, wo)
        dw[:, :, a, b] = np.einsum("nop,ncp->oc", dyf, xp[sl].reshape(n, c, ho * wo))
    return _unpad(dxp, pad), dw


def dwconv_vjp(x, w, stride, dy):
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    k = w.shape[1]
    pad = k // 2
    ho, wo = dy.shape[2], dy.shape[3]
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    for a, b, sl in _taps(k, stride, ho, wo):
        dxp[sl] += w[None, :, a, b, None, None] * dy
        dw[:, a, b] = (dy * xp[sl]).sum(axis=(0, 2, 3))
    return _unpad(dxp, pad), dw


def bn_act_vjp(x, gamma, beta, mean, var, eps, relu, dy):
    x, dy = _f64(x), _f64(dy)
    g, b, m, v = (_f64(t)[None, :, None, None] for t in (gamma, beta, mean, var))
    xhat = (x - m) / np.sqrt(v + eps)
    if relu:
        dy = dy * (g * xhat + b > 0.0)
    return dy * g / np.sqrt(v + eps), (dy * xhat).sum(axis=(0, 2, 3)), dy.sum(axis=(0, 2, 3))


def pool3x3_vjp(x, mode, stride, pad, dy):
    x, dy = _f64(x), _f64(dy)
    n, c, h, w = x.shape
    ho, wo = dy.shape[2], dy.shape[3]
    fill = -np.inf if mode == "max" else 0.0
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)), constant_values=fill)
    dxp = np.zeros_like(xp)
    if mode == "max":
        best = np.full((n, c, ho, wo), -np.inf)
        for a, b, sl in _taps(3, stride, ho, wo):
            best = np.maximum(best, xp[sl])
        taken = np.zeros((n, c, ho, wo), dtype=bool)
        for a, b, sl in _taps(3, stride, ho, wo):
            hit = (xp[sl] == best) & ~taken
            dxp[sl] += dy * hit
            taken |= hit
    else:
        ones = np.pad(np.ones((1, 1, h, w)), ((0, 0), (0, 0), (pad, pad), (pad, pad)))
        cnt = np.zeros((1, 1, ho, wo))
        for a, b, sl in _taps(3, stride, ho, wo):
            cnt = cnt + ones[sl]
        for a, b, sl in _taps(3, stride, ho, wo):
            dxp[sl] += dy / cnt * ones[sl]
    return _unpad(dxp, pad)


def node_vjp(nd, ins, dy) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    """(gradients w.r.t. the node's inputs, gradients w.r.t. its weight tensors)."""
    p, w = nd.params, nd.weights
    if nd.op == "conv1x1":
        dx, dw = conv2d_vjp(ins[0], _f64(w[0])[:, :, None, None], 1, 0, dy)
        return [dx], [dw[:, :, 0, 0]]
    if nd.op == "conv3x3":
        dx, dw = conv2d_vjp(ins[0], w[0], p["stride"], p["pad"], dy)
        return [dx], [dw]
    if nd.op == "dwconv":
        dx, dw = dwconv_vjp(ins[0], w[0], p["stride"], dy)
        return [dx], [dw]
    if nd.op == "bn_act":
        dx, dg, db = bn_act_vjp(ins[0], w[0], w[1], w[2], w[3], p["eps"], bool(p["relu"]), dy)
        return [dx], [dg, db, np.zeros_like(dg), np.zeros_like(dg)]
    if nd.op == "relu":
        return [_f64(dy) * (_f64(ins[0]) > 0.0)], []
    if nd.op == "add_n":
        return [_f64(dy).copy() for _ in ins], []
    if nd.op == "concat":
        out, first = [], 0
        for t, lo, hi in zip(ins, p["lo"], p["hi"]):
            d = np.zeros(t.shape)
            d[:, lo:hi] = _f64(dy)[:, first:first + hi - lo]
            first += hi - lo
            out.append(d)
        return out, []
    if nd.op == "pool":
        return [pool3x3_vjp(ins[0], p["mode"], p["stride"], p["pad"], dy)], []
    if nd.op == "global_avgpool":
        h, wd = ins[0].shape[2], ins[0].shape[3]
        return [np.broadcast_to(_f64(dy) / (h * wd), ins[0].shape).copy()], []
    if nd.op == "fc":
        x, dyf = _f64(ins[0]).reshape(ins[0].shape[0], -1), _f64(dy).reshape(dy.shape[0], -1)
        return [(dyf @ _f64(w[0])).reshape(ins[0].shape)], [dyf.T @ x, dyf.sum(axis=0)]
    raise ValueError(f"unknown op {nd.op!r}")


def backward(workload, seed: Dict[int, np.ndarray], x: Optional[np.ndarray] = None):
    """Returns (d_value, d_weight): d_value[v] = dL/d(value of node v) for every node,
    d_weight[v] = list of dL/d(weight j of node v), for L = sum_o <value[o], seed[o]>."""
    nodes = workload.nodes
    x = workload.input if x is None else x
    val: Dict[int, np.ndarray] = {}
    for v, nd in enumerate(nodes):
        val[v] = np.asarray(x) if nd.op == "input" else eval_node(nd, [val[u] for u in nd.preds])
    d_value = {v: np.zeros(val[v].shape) for v in range(len(nodes))}
    d_weight: Dict[int, List[np.ndarray]] = {}
    for o, s in seed.items():
        d_value[o] = d_value[o] + _f64(s)
    for v in range(len(nodes) - 1, -1, -1):
        nd = nodes[v]
        if nd.op == "input":
            continue
        dins, dws = node_vjp(nd, [val[u] for u in nd.preds], d_value[v])
        for u, d in zip(nd.preds, dins):          # a tensor read twice by one node gets both contributions
            d_value[u] = d_value[u] + d
        d_weight[v] = dws
    return d_value, d_weight


def sgd_step(weights: List[np.ndarray], grads: List[np.ndarray], lr: float) -> List[np.ndarray]:
    """Plain stochastic gradient descent: w <- w - lr * dL/dw, in fp64, stored as fp32."""
    return [np.ascontiguousarray(_f64(w) - lr * _f64(g), dtype=np.float32) for w, g in zip(weights, grads)]
