"""Whole-DAG evaluation for the oracle (test infrastructure, see package doc).

Section 4.1 of the paper: ahead-of-time scheduling moves work out of the run
loop without changing what the network computes. The reference result is
therefore the DAG evaluated one node at a time in ascending id order.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional

import numpy as np

from . import ops


def eval_node(nd, ins):
    p, w = nd.params, nd.weights
    if nd.op == "conv1x1":
        return ops.conv1x1(ins[0], w[0])
    if nd.op == "dwconv":
        return ops.dwconv(ins[0], w[0], p["stride"])
    if nd.op == "conv3x3":
        return ops.conv3x3(ins[0], w[0], p["stride"], p["pad"])
    if nd.op == "bn_act":
        return ops.bn_act(ins[0], w[0], w[1], w[2], w[3], p["eps"], bool(p["relu"]))
    if nd.op == "relu":
        return ops.relu(ins[0])
    if nd.op == "add_n":
        return ops.add_n(ins)
    if nd.op == "concat":
        return ops.concat(ins, p["lo"], p["hi"])
    if nd.op == "pool":
        return ops.pool3x3(ins[0], p["mode"], p["stride"], p["pad"])
    if nd.op == "global_avgpool":
        return ops.global_avgpool(ins[0])
    if nd.op == "fc":
        return ops.fc(ins[0], w[0], w[1])
    raise ValueError(f"unknown op {nd.op!r}")


def forward(workload, x: Optional[np.ndarray] = None, keep: Optional[Iterable[int]] = None) -> Dict[int, np.ndarray]:
    """Evaluate every node; return {id: fp32 array} for ``keep`` (default: the
    workload's outputs; pass ``range(len(nodes))`` for every tensor)."""
    nodes = workload.nodes
    x = workload.input if x is None else x
    keep = set(workload.outputs if keep is None else keep)
    last_use = {}
    for v, nd in enumerate(nodes):
        for u in nd.preds:
            last_use[u] = v
    val: Dict[int, np.ndarray] = {}
    out: Dict[int, np.ndarray] = {}
    for v, nd in enumerate(nodes):
        if nd.op == "input":
            assert tuple(x.shape) == (nd.params["n"], nd.params["c"], nd.params["h"], nd.params["w"])
            val[v] = np.ascontiguousarray(x, dtype=np.float32)
        else:
            val[v] = eval_node(nd, [val[u] for u in nd.preds])
        if v in keep:
            out[v] = val[v]
        for u in set(nd.preds):            # drop tensors nobody reads any more
            if last_use[u] == v:
                del val[u]
    return out
