"""The DAG of one training iteration, derived from a forward workload (structure only).

Section 5 of the paper (training results) replays a whole iteration - forward pass, backward
pass and weight update - as one recorded schedule. This module writes that iteration down as
a DAG in the same vocabulary as the inference workloads: the forward nodes keep their ids, one
extra input node per network output carries dL/d(output) (the "seed": the loss is
L = sum_o <value[o], seed[o]>), then, walking the forward nodes in descending id, one node per
backward operator, an ``add_n`` wherever a tensor has several readers, and one ``sgd_update``
node per weight tensor. It performs no arithmetic: what each operator computes is the business
of whoever executes the DAG.

Backward operator vocabulary ("dy" = gradient w.r.t. the forward operator's result, "x" = the
forward operator's input; weights are shared with the forward node):

    conv1x1_dgrad         preds [dy]       cout = channels of x          shared W
    conv1x1_wgrad         preds [dy, x]                                   -> [cout, cin, 1, 1]
    conv3x3_dgrad / _wgrad preds [dy, x]   stride, pad                    shared W (dgrad)
    dwconv_dgrad / _wgrad  preds [dy, x]   k, stride                      shared W (dgrad); wgrad -> [1, c, k, k]
    bn_act_dgrad / _wgrad  preds [dy, x]   eps, relu                      shared gamma, beta, mean, var; wgrad -> [2, c, 1, 1]
    relu_dgrad, pool_dgrad (mode, stride, pad), global_avgpool_dgrad      preds [dy, x]
    channel_sum           preds [dy]                                      -> [1, c, 1, 1]  (fc bias gradient)
    slice_pad             preds [dy]       cout, src_lo, src_hi, dst_lo   (gradient of one concat input)
    sgd_update            preds [grad, the other readers of the weight: its backward operator, its forward node]
                          lr, offset, numel                                shared W (written in place)
    the fc uses conv1x1_dgrad / conv1x1_wgrad on its [n, c, 1, 1] tensors
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from .model import Node, Workload


@dataclass
class TrainingWorkload(Workload):
    forward: Workload = None
    lr: float = 0.0
    inputs: Dict[int, np.ndarray] = field(default_factory=dict)      # input node id -> value (x and the seeds)
    seed_of: Dict[int, int] = field(default_factory=dict)            # forward output -> its seed input node
    grad_of: Dict[int, int] = field(default_factory=dict)            # forward node -> node holding dL/d(its value)
    wgrad_of: Dict[Tuple[int, int], Tuple[int, int, int]] = field(default_factory=dict)   # (forward node, weight j) -> (node, offset, numel)
    update_of: Dict[Tuple[int, int], int] = field(default_factory=dict)


def training_graph(fwd: Workload, lr: float, seeds: Dict[int, np.ndarray]) -> TrainingWorkload:
    nodes: List[Node] = [Node(nd.op, list(nd.preds), dict(nd.params), nd.weights, nd.shape, nd.init_gain) for nd in fwd.nodes]
    n_fwd = len(nodes)

    def add(op, preds, shape, shared=(), **params) -> int:
        nodes.append(Node(op, list(preds), dict(params), [], tuple(int(s) for s in shape), 1.0, list(shared)))
        return len(nodes) - 1

    inputs = {0: fwd.input}
    seed_of, grad_of, wgrad_of, update_of = {}, {}, {}, {}
    contrib: Dict[int, List[int]] = {v: [] for v in range(n_fwd)}
    for o in sorted(seeds):
        s = add("input", [], fwd.nodes[o].shape, n=fwd.nodes[o].shape[0], c=fwd.nodes[o].shape[1], h=fwd.nodes[o].shape[2], w=fwd.nodes[o].shape[3])
        inputs[s] = np.ascontiguousarray(seeds[o], dtype=np.float32)
        seed_of[o] = s
        contrib[o].append(s)
    needs_grad = [nd.op != "input" for nd in fwd.nodes]

    def update(v, j, grad_node, offset, numel, after):
        # the update writes the weight in place: every reader of the weight must have run - the backward operator
        # that reads it and the forward node itself (whose result need not be an ancestor of the gradient: the
        # gradient of a network output comes straight from the seed)
        preds = [grad_node] + [a for a in after if a is not None] + [v]
        update_of[(v, j)] = add("sgd_update", preds, (1, 1, 1, 1), shared=[(v, j)], lr=float(lr), offset=int(offset), numel=int(numel))
        wgrad_of[(v, j)] = (grad_node, int(offset), int(numel))

    for v in range(n_fwd - 1, -1, -1):
        nd = fwd.nodes[v]
        if nd.op == "input" or not contrib[v]:
            continue
        c = contrib[v]
        while len(c) > 8:                                   # an operator takes at most 8 predecessors
            c = [add("add_n", c[:8], nd.shape)] + c[8:]
        dy = c[0] if len(c) == 1 else add("add_n", c, nd.shape)
        grad_of[v] = dy
        p = nd.params
        x = nd.preds[0]
        xs = fwd.nodes[x].shape
        want_dx = needs_grad[x]
        if nd.op in ("conv1x1", "fc"):
            dx = add("conv1x1_dgrad", [dy], xs, shared=[(v, 0)], cout=xs[1]) if want_dx else None
            wg = add("conv1x1_wgrad", [dy, x], (nd.shape[1], xs[1], 1, 1))
            update(v, 0, wg, 0, nd.shape[1] * xs[1], [dx])
            if nd.op == "fc":
                bs = add("channel_sum", [dy], (1, nd.shape[1], 1, 1))
                update(v, 1, bs, 0, nd.shape[1], [])
            if want_dx:
                contrib[x].append(dx)
        elif nd.op == "conv3x3":
            dx = add("conv3x3_dgrad", [dy, x], xs, shared=[(v, 0)], stride=p["stride"], pad=p["pad"]) if want_dx else None
            wg = add("conv3x3_wgrad", [dy, x], (nd.shape[1], xs[1], 3, 3), stride=p["stride"], pad=p["pad"])
            update(v, 0, wg, 0, nd.shape[1] * xs[1] * 9, [dx])
            if want_dx:
                contrib[x].append(dx)
        elif nd.op == "dwconv":
            dx = add("dwconv_dgrad", [dy, x], xs, shared=[(v, 0)], k=p["k"], stride=p["stride"]) if want_dx else None
            wg = add("dwconv_wgrad", [dy, x], (1, xs[1], p["k"], p["k"]), k=p["k"], stride=p["stride"])
            update(v, 0, wg, 0, xs[1] * p["k"] * p["k"], [dx])
            if want_dx:
                contrib[x].append(dx)
        elif nd.op == "bn_act":
            four = [(v, j) for j in range(4)]
            dx = add("bn_act_dgrad", [dy, x], xs, shared=four, eps=p["eps"], relu=p["relu"]) if want_dx else None
            wg = add("bn_act_wgrad", [dy, x], (2, xs[1], 1, 1), shared=four, eps=p["eps"], relu=p["relu"])
            update(v, 0, wg, 0, xs[1], [dx])                # gamma
            update(v, 1, wg, xs[1], xs[1], [dx])            # beta
            if want_dx:
                contrib[x].append(dx)
        elif nd.op == "relu":
            if want_dx:
                contrib[x].append(add("relu_dgrad", [dy, x], xs))
        elif nd.op == "pool":
            if want_dx:
                contrib[x].append(add("pool_dgrad", [dy, x], xs, mode=p["mode"], stride=p["stride"], pad=p["pad"]))
        elif nd.op == "global_avgpool":
            if want_dx:
                contrib[x].append(add("global_avgpool_dgrad", [dy, x], xs))
        elif nd.op == "add_n":
            for u in nd.preds:
                if needs_grad[u]:
                    contrib[u].append(dy)
        elif nd.op == "concat":
            first = 0
            for u, lo, hi in zip(nd.preds, p["lo"], p["hi"]):
                if needs_grad[u]:
                    us = fwd.nodes[u].shape
                    contrib[u].append(add("slice_pad", [dy], us, cout=us[1], src_lo=first, src_hi=first + hi - lo, dst_lo=lo))
                first += hi - lo
        else:
            raise ValueError(f"no backward rule for {nd.op!r}")
    outputs = sorted(set(fwd.outputs) | set(update_of.values()))
    return TrainingWorkload(fwd.name + "_training", nodes, fwd.input, outputs, forward=fwd, lr=float(lr), inputs=inputs,
                            seed_of=seed_of, grad_of=grad_of, wgrad_of=wgrad_of, update_of=update_of)


def nas_cell_cifar(seed: int = 0, batch: int = 32, c: int = 44, image: int = 32, n_classes: int = 10) -> Workload:
    """Forward network of the training workload: a 3x3 stem, one normal and one reduction cell of the
    NASNet-style recipe (drawn from the same generator as the inference configuration), ReLU, global
    average pool and a 10-way fc, on CIFAR-sized inputs [batch, 3, 32, 32] ~ N(0, 1)."""
    from .configs import _cell, _draw_cell
    from .model import Builder
    rng = np.random.default_rng(seed)
    normal = _draw_cell(rng, False)
    reduce_ = _draw_cell(rng, True)
    b = Builder("nas_cell_cifar")
    x = b.input(batch, 3, image, image)
    x = b.conv3x3(x, c, 1, 1)
    x = b.bn_act(x, relu=True)
    prev = prevprev = x
    prev, prevprev = _cell(b, prev, prevprev, c, normal, False), prev
    prev, prevprev = _cell(b, prev, prevprev, 2 * c, reduce_, True), prev
    x = b.relu(prev)
    x = b.global_avgpool(x)
    b.fc(x, n_classes)
    b.draw_weights(rng, "he", "random")
    return b.finish(rng)
