"""Recipes for the five benchmark configurations (all seeded, all synthetic).

Each recipe draws, in this order and from one ``numpy.random.default_rng(seed)``
stream: the topology (where it is random), then the weights in ascending node
id, then the input tensor.
"""
from __future__ import annotations

import numpy as np

from .model import Builder, Workload

CONFIG_NAMES = ("tiny_cell", "chain50", "random200", "nasnet_style", "inception_style")


# ---------------------------------------------------------------------------
# 1. tiny two-branch cell: 8 nodes (input + 7 tasks), two concurrent branches
# ---------------------------------------------------------------------------
def tiny_cell(seed: int = 0) -> Workload:
    rng = np.random.default_rng(seed)
    b = Builder("tiny_cell")
    x = b.input(1, 16, 8, 8)
    a = b.conv1x1(x, 16)            # branch A: 1x1 conv, BN, ReLU (BN and ReLU as two tasks)
    a = b.bn_act(a, relu=False)
    a = b.relu(a)
    c = b.dwconv(x, 3, 1)           # branch B: 3x3 depthwise, 1x1 conv, BN
    c = b.conv1x1(c, 16)
    c = b.bn_act(c, relu=False)
    b.add_n([a, c])
    b.draw_weights(rng, 0.1, "identity")
    return b.finish(rng)


# ---------------------------------------------------------------------------
# 2. linear chain: 50 x [conv3x3 32->32 pad 1, BN+ReLU]
# ---------------------------------------------------------------------------
def chain50(seed: int = 0, blocks: int = 50) -> Workload:
    rng = np.random.default_rng(seed)
    b = Builder("chain50")
    x = b.input(1, 32, 32, 32)
    for _ in range(blocks):
        x = b.conv3x3(x, 32, 1, 1)
        x = b.bn_act(x, relu=True)
    b.draw_weights(rng, "he", "identity")
    return b.finish(rng)


# ---------------------------------------------------------------------------
# 3. random layered DAG: 200 operator nodes in 20 layers of width 1..16
# ---------------------------------------------------------------------------
def random_layered(seed: int = 0, n_nodes: int = 200, n_layers: int = 20,
                   max_width: int = 16, shape=(1, 64, 28, 28), name="random200") -> Workload:
    rng = np.random.default_rng(seed)
    widths = rng.integers(1, max_width + 1, n_layers)
    while widths.sum() != n_nodes:          # nudge random layers until the total fits
        i = int(rng.integers(0, n_layers))
        step = 1 if widths.sum() < n_nodes else -1
        if 1 <= widths[i] + step <= max_width:
            widths[i] += step
    b = Builder(name)
    x = b.input(*shape)
    c = shape[1]
    earlier: list[int] = []                 # operator nodes of all earlier layers
    for li in range(n_layers):
        this_layer = []
        for _ in range(int(widths[li])):
            if li == 0:
                preds = [x]
            else:
                k = min(int(rng.integers(1, 4)), len(earlier))
                preds = sorted(int(p) for p in rng.choice(earlier, size=k, replace=False))
            if len(preds) == 1:
                kind = int(rng.integers(0, 3))
                if kind == 0:
                    v = b.conv1x1(preds[0], c)
                elif kind == 1:
                    v = b.dwconv(preds[0], 3, 1)
                else:
                    v = b.bn_act(preds[0], relu=True)
            elif int(rng.integers(0, 2)) == 0:
                v = b.add_n(preds)
            else:                           # channel block j comes from predecessor j
                k = len(preds)
                blk = -(-c // k)
                slices = [(j * blk, min(c, (j + 1) * blk)) for j in range(k)]
                v = b.concat(preds, slices)
            this_layer.append(v)
        earlier.extend(this_layer)
    b.draw_weights(rng, 0.05, "random")
    return b.finish(rng)


# ---------------------------------------------------------------------------
# 4. NASNet-A-style stack: 12 normal cells + 2 reduction cells
# ---------------------------------------------------------------------------
_CELL_OPS = ("sep3", "sep5", "avg", "max", "id")


def _draw_cell(rng, reduction: bool, n_blocks: int = 5):
    """Five blocks; block i combines two earlier hidden states (0, 1 = the two
    adjusted cell inputs, 2 + j = block j) through two branch operators. A cell
    input is three times as likely to be picked as an earlier block, which gives
    the wide, shallow cells typical of searched architectures."""
    blocks = []
    for i in range(n_blocks):
        p = np.array([3.0, 3.0] + [1.0] * i)
        p /= p.sum()
        while True:
            src = [int(s) for s in rng.choice(i + 2, size=2, p=p)]
            ops = [_CELL_OPS[int(o)] for o in rng.integers(0, len(_CELL_OPS), 2)]
            if ops[0] == "id" and ops[1] == "id":
                continue
            if reduction and any(o == "id" and s < 2 for o, s in zip(ops, src)):
                continue                    # a cell input must be strided in a reduction cell
            break
        blocks.append((src, ops))
    return blocks


def _sep(b: Builder, x: int, k: int, stride: int, c: int) -> int:
    for s in (stride, 1):                   # depthwise + pointwise + BN + ReLU, twice
        x = b.dwconv(x, k, s)
        x = b.conv1x1(x, c)
        x = b.bn_act(x, relu=True)
    return x


def _branch(b: Builder, x: int, op: str, stride: int, c: int) -> int:
    if op == "sep3":
        return _sep(b, x, 3, stride, c)
    if op == "sep5":
        return _sep(b, x, 5, stride, c)
    if op in ("avg", "max"):
        return b.pool(x, op, stride, 1)
    assert op == "id" and stride == 1
    return x


def _cell(b: Builder, prev: int, prevprev: int, c: int, spec, reduction: bool) -> int:
    hw = b.shape(prev)[2]
    hidden = []
    for h in (prev, prevprev):              # bring both cell inputs to c channels at prev's size
        if b.shape(h)[2] != hw:
            h = b.pool(h, "avg", 2, 1)
        h = b.conv1x1(h, c, init_gain=0.3)   # keeps activations O(1..100) through 14 cells
        h = b.bn_act(h, relu=False)
        hidden.append(h)
    consumed = set()
    for src, ops in spec:
        outs = []
        for s, o in zip(src, ops):
            stride = 2 if (reduction and s < 2) else 1
            outs.append(_branch(b, hidden[s], o, stride, c))
            consumed.add(s)
        hidden.append(b.add_n(outs))
    free = [hidden[i] for i in range(2, len(hidden)) if i not in consumed]
    return free[0] if len(free) == 1 else b.concat(free)


def nasnet_style(seed: int = 0, cells_per_stage: int = 4, c0: int = 44,
                 image: int = 224, n_classes: int = 1000) -> Workload:
    rng = np.random.default_rng(seed)
    normal = _draw_cell(rng, False)
    reduce_ = _draw_cell(rng, True)
    b = Builder("nasnet_style")
    x = b.input(1, 3, image, image)
    x = b.conv3x3(x, c0, 2, 1)
    x = b.bn_act(x, relu=True)
    x = b.pool(x, "max", 2, 1)
    x = b.pool(x, "max", 2, 1)
    prev = prevprev = x
    c = c0
    for stage in range(3):
        if stage > 0:
            c *= 2
            prev, prevprev = _cell(b, prev, prevprev, c, reduce_, True), prev
        for _ in range(cells_per_stage):
            prev, prevprev = _cell(b, prev, prevprev, c, normal, False), prev
    x = b.relu(prev)
    x = b.global_avgpool(x)
    b.fc(x, n_classes)
    b.draw_weights(rng, "he", "random")
    return b.finish(rng)


# ---------------------------------------------------------------------------
# 5. Inception-v3-style network (four-branch blocks, conv + BN/ReLU, concat)
# ---------------------------------------------------------------------------
def _cbr1(b: Builder, x: int, cout: int) -> int:
    return b.bn_act(b.conv1x1(x, cout), relu=True)


def _cbr3(b: Builder, x: int, cout: int, stride: int = 1, pad: int = 1) -> int:
    return b.bn_act(b.conv3x3(x, cout, stride, pad), relu=True)


def _block4(b: Builder, x: int, c1: int, c2: tuple, c3: tuple, c4: int) -> int:
    b1 = _cbr1(b, x, c1)
    b2 = _cbr3(b, _cbr1(b, x, c2[0]), c2[1])
    b3 = _cbr3(b, _cbr3(b, _cbr1(b, x, c3[0]), c3[1]), c3[2])
    b4 = _cbr1(b, b.pool(x, "avg", 1, 1), c4)
    return b.concat([b1, b2, b3, b4])


def inception_style(seed: int = 0, batch: int = 1, image: int = 299,
                    n_classes: int = 1000) -> Workload:
    rng = np.random.default_rng(seed)
    b = Builder("inception_style")
    x = b.input(batch, 3, image, image)
    x = _cbr3(b, x, 32, 2, 0)
    x = _cbr3(b, x, 32, 1, 0)
    x = _cbr3(b, x, 64, 1, 1)
    x = b.pool(x, "max", 2, 0)
    x = _cbr1(b, x, 80)
    x = _cbr3(b, x, 192, 1, 0)
    x = b.pool(x, "max", 2, 0)
    for c4 in (32, 64, 64):                                  # 35 x 35 blocks
        x = _block4(b, x, 64, (48, 64), (64, 96, 96), c4)
    r1 = _cbr3(b, x, 384, 2, 0)                              # grid reduction to 17 x 17
    r2 = _cbr3(b, _cbr3(b, _cbr1(b, x, 64), 96), 96, 2, 0)
    x = b.concat([r1, r2, b.pool(x, "max", 2, 0)])
    for m in (128, 160, 160, 192):                           # 17 x 17 blocks
        x = _block4(b, x, 192, (m, 192), (m, m, 192), 192)
    r1 = _cbr3(b, _cbr1(b, x, 192), 320, 2, 0)               # grid reduction to 8 x 8
    r2 = _cbr3(b, _cbr3(b, _cbr1(b, x, 192), 192), 192, 2, 0)
    x = b.concat([r1, r2, b.pool(x, "max", 2, 0)])
    for _ in range(2):                                       # 8 x 8 blocks, 2048 channels out
        x = _block4(b, x, 320, (384, 768), (448, 384, 768), 192)
    x = b.global_avgpool(x)
    b.fc(x, n_classes)
    b.draw_weights(rng, "he", "random")
    return b.finish(rng)


def make(name: str, seed: int = 0, **kw) -> Workload:
    """Build one of CONFIG_NAMES (extra keywords go to the recipe, e.g. batch=32)."""
    table = {"tiny_cell": tiny_cell, "chain50": chain50, "random200": random_layered,
             "nasnet_style": nasnet_style, "inception_style": inception_style}
    return table[name](seed, **kw)
