"""Seeded synthetic operator DAGs (the five benchmark configurations).

This package only *describes* workloads: node list, op names, integer/float
parameters, predecessor ids, and randomly drawn fp32 weight and input arrays.
It performs none of the arithmetic of the operators and none of the scheduling;
the CPU oracle and the HIP library each read these descriptions and do their
own shape inference, scheduling and computation.

Conventions shared by every consumer (an interface, not an implementation):

* node ids are list positions; predecessors always have smaller ids, so the
  ascending id order is a topological order (node 0 is the single input node);
* tensors are fp32, NCHW;
* op vocabulary and parameters:
    input           n, c, h, w
    conv1x1         cout                    weights: W[cout, cin]
    dwconv          k (3|5), stride (1|2)   weights: W[c, k, k]; pad = k // 2
    conv3x3         cout, stride, pad       weights: W[cout, cin, 3, 3]
    bn_act          eps, relu (0|1)         weights: gamma, beta, mean, var  [c]
    relu            -
    add_n           -                       2..8 predecessors of equal shape
    concat          lo[], hi[]              channel slice [lo_j, hi_j) of pred j,
                                            slices stacked along C in pred order
    pool            mode ('max'|'avg'), stride (1|2), pad (0|1); window 3x3;
                    avg divides by the number of in-bounds taps, max ignores
                    out-of-bounds taps
    global_avgpool  -                       -> [n, c, 1, 1]
    fc              cout                    weights: W[cout, cin], b[cout];
                                            input must be [n, cin, 1, 1]
"""
from .model import Node, Workload, OPS, TRAIN_OPS  # noqa: F401
from .configs import make, CONFIG_NAMES  # noqa: F401
from .training import training_graph, nas_cell_cifar, TrainingWorkload  # noqa: F401
