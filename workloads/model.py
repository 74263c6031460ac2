"""Workload description records and the builder the config recipes use."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

OPS = ("input", "conv1x1", "dwconv", "conv3x3", "bn_act", "relu", "add_n",
       "concat", "pool", "global_avgpool", "fc")
# operators that only occur in the DAG of a training iteration (see workloads/training.py)
TRAIN_OPS = ("conv1x1_dgrad", "conv1x1_wgrad", "conv3x3_dgrad", "conv3x3_wgrad", "dwconv_dgrad", "dwconv_wgrad",
             "bn_act_dgrad", "bn_act_wgrad", "relu_dgrad", "pool_dgrad", "global_avgpool_dgrad", "channel_sum",
             "slice_pad", "sgd_update")


@dataclass
class Node:
    op: str
    preds: List[int]
    params: Dict[str, object] = field(default_factory=dict)
    weights: List[np.ndarray] = field(default_factory=list)
    # Shape the recipe expects for this node's output. Consumers infer shapes
    # themselves; tests compare their result with this field.
    shape: Tuple[int, int, int, int] = (0, 0, 0, 0)
    # Multiplier on the std of this node's random weights (recipe-internal).
    init_gain: float = 1.0
    # Weight buffers this node shares with earlier nodes, as (node id, weight index) pairs, in the order the
    # operator takes them (a backward operator reads the forward operator's weights, the update writes them).
    shared_weights: List[Tuple[int, int]] = field(default_factory=list)


@dataclass
class Workload:
    name: str
    nodes: List[Node]
    input: np.ndarray          # fp32 [n, c, h, w], the value of node 0
    outputs: List[int]         # ids whose tensors are compared / returned

    @property
    def edges(self) -> List[Tuple[int, int]]:
        """Distinct dependency edges (u, v), sorted."""
        return sorted({(u, v) for v, nd in enumerate(self.nodes) for u in nd.preds})


def _out_hw(h: int, w: int, k: int, stride: int, pad: int) -> Tuple[int, int]:
    return (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1


class Builder:
    """Appends nodes and keeps the expected output shape of each one so that
    weight arrays can be sized. Weight *values* are drawn later, in node-id
    order, by ``draw_weights`` (draw order: topology, weights, input)."""

    def __init__(self, name: str):
        self.name = name
        self.nodes: List[Node] = []

    # -- structure -----------------------------------------------------
    def _add(self, op, preds, shape, **params) -> int:
        for p in preds:
            assert 0 <= p < len(self.nodes)
        self.nodes.append(Node(op, list(preds), dict(params), [], tuple(int(s) for s in shape)))
        return len(self.nodes) - 1

    def shape(self, i: int):
        return self.nodes[i].shape

    def input(self, n, c, h, w) -> int:
        assert not self.nodes
        return self._add("input", [], (n, c, h, w), n=n, c=c, h=h, w=w)

    def conv1x1(self, x, cout, init_gain: float = 1.0) -> int:
        n, c, h, w = self.shape(x)
        v = self._add("conv1x1", [x], (n, cout, h, w), cout=cout)
        self.nodes[v].init_gain = float(init_gain)
        return v

    def dwconv(self, x, k, stride=1) -> int:
        n, c, h, w = self.shape(x)
        ho, wo = _out_hw(h, w, k, stride, k // 2)
        return self._add("dwconv", [x], (n, c, ho, wo), k=k, stride=stride)

    def conv3x3(self, x, cout, stride=1, pad=1) -> int:
        n, c, h, w = self.shape(x)
        ho, wo = _out_hw(h, w, 3, stride, pad)
        return self._add("conv3x3", [x], (n, cout, ho, wo), cout=cout, stride=stride, pad=pad)

    def bn_act(self, x, relu=True, eps=1e-5) -> int:
        return self._add("bn_act", [x], self.shape(x), eps=float(eps), relu=int(bool(relu)))

    def relu(self, x) -> int:
        return self._add("relu", [x], self.shape(x))

    def add_n(self, xs) -> int:
        assert 2 <= len(xs) <= 8          # the library takes up to 8 predecessors per node
        s = self.shape(xs[0])
        assert all(self.shape(x) == s for x in xs), [self.shape(x) for x in xs]
        return self._add("add_n", xs, s)

    def concat(self, xs, slices=None) -> int:
        n, _, h, w = self.shape(xs[0])
        if slices is None:
            slices = [(0, self.shape(x)[1]) for x in xs]
        ctot = 0
        for x, (lo, hi) in zip(xs, slices):
            sn, sc, sh, sw = self.shape(x)
            assert (sn, sh, sw) == (n, h, w) and 0 <= lo < hi <= sc
            ctot += hi - lo
        return self._add("concat", xs, (n, ctot, h, w),
                         lo=[int(s[0]) for s in slices], hi=[int(s[1]) for s in slices])

    def pool(self, x, mode, stride=1, pad=1) -> int:
        assert mode in ("max", "avg")
        n, c, h, w = self.shape(x)
        ho, wo = _out_hw(h, w, 3, stride, pad)
        return self._add("pool", [x], (n, c, ho, wo), mode=mode, stride=stride, pad=pad)

    def global_avgpool(self, x) -> int:
        n, c, _, _ = self.shape(x)
        return self._add("global_avgpool", [x], (n, c, 1, 1))

    def fc(self, x, cout) -> int:
        n, c, h, w = self.shape(x)
        assert h == 1 and w == 1
        return self._add("fc", [x], (n, cout, 1, 1), cout=cout)

    # -- values --------------------------------------------------------
    def draw_weights(self, rng: np.random.Generator, conv_std, bn_mode: str):
        """Fill weights in ascending node id.

        conv_std: float (fixed std) or 'he' (std = sqrt(2 / fan_in)).
        bn_mode: 'identity' (gamma 1, beta 0, mean 0, var 1) or 'random'
                 (gamma~U(.8,1.2), beta~N(0,.1), mean~N(0,.1), var~U(.8,1.2)).
        """
        def normal(shape, fan_in):
            std = np.sqrt(2.0 / fan_in) if conv_std == "he" else float(conv_std)
            return (rng.standard_normal(shape) * (std * nd.init_gain)).astype(np.float32)

        for nd in self.nodes:
            if nd.op == "conv1x1":
                cin = self.shape(nd.preds[0])[1]
                nd.weights = [normal((nd.params["cout"], cin), cin)]
            elif nd.op == "dwconv":
                c, k = nd.shape[1], nd.params["k"]
                nd.weights = [normal((c, k, k), k * k)]
            elif nd.op == "conv3x3":
                cin = self.shape(nd.preds[0])[1]
                nd.weights = [normal((nd.params["cout"], cin, 3, 3), cin * 9)]
            elif nd.op == "fc":
                cin = self.shape(nd.preds[0])[1]
                nd.weights = [normal((nd.params["cout"], cin), cin),
                              (rng.standard_normal(nd.params["cout"]) * 0.01).astype(np.float32)]
            elif nd.op == "bn_act":
                c = nd.shape[1]
                if bn_mode == "identity":
                    nd.weights = [np.ones(c, np.float32), np.zeros(c, np.float32),
                                  np.zeros(c, np.float32), np.ones(c, np.float32)]
                else:
                    nd.weights = [rng.uniform(0.8, 1.2, c).astype(np.float32),
                                  (rng.standard_normal(c) * 0.1).astype(np.float32),
                                  (rng.standard_normal(c) * 0.1).astype(np.float32),
                                  rng.uniform(0.8, 1.2, c).astype(np.float32)]

    def finish(self, rng: np.random.Generator, outputs=None) -> Workload:
        x = rng.standard_normal(self.nodes[0].shape).astype(np.float32)
        if outputs is None:  # every sink
            used = {p for nd in self.nodes for p in nd.preds}
            outputs = [i for i in range(len(self.nodes)) if i not in used]
        return Workload(self.name, self.nodes, x, list(outputs))
