"""Pins of the oracle's backward pass (oracle/backward.py; Section 5 of the paper, training):
central finite differences of an fp64 forward pass on small DAGs that use every operator,
torch.autograd (CPU, fp64) operator by operator, and closed forms."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ops
from oracle.backward import backward, node_vjp, sgd_step
from oracle.forward import eval_node
from workloads.model import Builder


@pytest.fixture
def fp64_storage(monkeypatch):
    # the forward oracle stores fp32 between operators; derivatives are checked on the same
    # formulas evaluated in fp64 throughout
    monkeypatch.setattr(ops, "_out", lambda x: np.ascontiguousarray(x, dtype=np.float64))


def _cell(b):
    x = b.input(2, 6, 9, 8)
    a = b.bn_act(b.conv1x1(x, 8), relu=True)
    c = b.conv3x3(b.dwconv(a, 3, 1), 8, 1, 1)
    d = b.bn_act(b.conv3x3(x, 8, 1, 1), relu=False)
    e = b.add_n([a, c, d, a])                                   # one tensor read twice by one node
    f = b.pool(e, "avg", 1, 1)
    g = b.pool(b.relu(e), "max", 2, 1)
    h = b.conv3x3(f, 5, 2, 1)
    i = b.dwconv(b.conv3x3(f, 5, 2, 1), 5, 1)
    j = b.concat([g, h, b.pool(i, "max", 1, 1)], slices=[(2, 7), (0, 5), (1, 4)])
    b.fc(b.global_avgpool(j), 7)
    b.dwconv(j, 3, 2)


def _workload(build=_cell, seed=3):
    b = Builder("grad")
    build(b)
    rng = np.random.default_rng(seed)
    b.draw_weights(rng, 0.3, "random")
    return b.finish(rng)


def _values(w):
    # the DAG in ascending id like oracle.forward, but without its fp32 copy of the input
    val = {}
    for v, nd in enumerate(w.nodes):
        val[v] = np.asarray(w.input, dtype=np.float64) if nd.op == "input" else eval_node(nd, [val[u] for u in nd.preds])
    return val


def _loss(w, seed):
    val = _values(w)
    return sum(float((np.asarray(val[o], dtype=np.float64) * s).sum()) for o, s in seed.items())


def test_gradients_match_central_differences(fp64_storage):
    w = _workload()
    w.input = np.asarray(w.input, dtype=np.float64)
    for nd in w.nodes:
        nd.weights = [np.asarray(t, dtype=np.float64) for t in nd.weights]
    rng = np.random.default_rng(5)
    sinks = [v for v in range(len(w.nodes)) if all(v not in nd.preds for nd in w.nodes)]
    assert len(sinks) == 2
    seed = {o: rng.standard_normal(_values(w)[o].shape) for o in sinks}
    d_value, d_weight = backward(w, seed)
    h = 1e-5

    def check(array, grad, what):
        flat, g = array.reshape(-1), np.asarray(grad).reshape(-1)
        for idx in rng.choice(flat.size, size=min(6, flat.size), replace=False):
            keep = flat[idx]
            flat[idx] = keep + h
            up = _loss(w, seed)
            flat[idx] = keep - h
            down = _loss(w, seed)
            flat[idx] = keep
            fd = (up - down) / (2 * h)
            assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd)), (what, idx, fd, g[idx])

    check(w.input, d_value[0], "input")
    for v, nd in enumerate(w.nodes):
        for j, t in enumerate(nd.weights):
            if nd.op == "bn_act" and j >= 2:
                assert not d_weight[v][j].any()                  # statistics are fixed
                continue
            check(t, d_weight[v][j], (v, nd.op, j))


def _t(a):
    return torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (2, 0), (1, 0)])
def test_conv_and_pool_vjps_match_torch_autograd(stride, pad):
    rng = np.random.default_rng(stride * 10 + pad)
    x = rng.standard_normal((2, 5, 9, 11))

    class N:                                                      # the fields node_vjp reads
        def __init__(self, op, params, weights):
            self.op, self.params, self.weights = op, params, weights

    w3 = rng.standard_normal((4, 5, 3, 3))
    xt, wt = _t(x), _t(w3)
    y = F.conv2d(xt, wt, stride=stride, padding=pad)
    dy = rng.standard_normal(tuple(y.shape))
    y.backward(torch.tensor(dy))
    (dx,), (dw,) = node_vjp(N("conv3x3", {"stride": stride, "pad": pad}, [w3]), [x], dy)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12) and np.allclose(dw, wt.grad.numpy(), atol=1e-12)

    for k in (3, 5):
        wd = rng.standard_normal((5, k, k))
        xt, wt = _t(x), _t(wd[:, None])
        y = F.conv2d(xt, wt, stride=stride, padding=k // 2, groups=5)
        dy = rng.standard_normal(tuple(y.shape))
        y.backward(torch.tensor(dy))
        (dx,), (dw,) = node_vjp(N("dwconv", {"stride": stride}, [wd]), [x], dy)
        assert np.allclose(dx, xt.grad.numpy(), atol=1e-12) and np.allclose(dw, wt.grad.numpy()[:, 0], atol=1e-12)

    if pad <= 1:
        for mode in ("max", "avg"):
            xt = _t(x)
            y = (F.max_pool2d(xt, 3, stride, pad) if mode == "max"
                 else F.avg_pool2d(xt, 3, stride, pad, count_include_pad=False))
            dy = rng.standard_normal(tuple(y.shape))
            y.backward(torch.tensor(dy))
            (dx,), _ = node_vjp(N("pool", {"mode": mode, "stride": stride, "pad": pad}, []), [x], dy)
            assert np.allclose(dx, xt.grad.numpy(), atol=1e-12), mode


def test_closed_forms_and_the_update():
    rng = np.random.default_rng(1)

    class N:
        def __init__(self, op, params, weights):
            self.op, self.params, self.weights = op, params, weights

    dy = rng.standard_normal((2, 7, 3, 4))
    xs = [rng.standard_normal((2, 7, 3, 4)) for _ in range(3)]
    dins, dws = node_vjp(N("add_n", {}, []), xs, dy)
    assert len(dins) == 3 and all(np.array_equal(d, dy) for d in dins) and dws == []
    # a concat's gradient is the matching slice, zero outside the slice it took
    a, b = rng.standard_normal((2, 6, 3, 4)), rng.standard_normal((2, 5, 3, 4))
    (da, db), _ = node_vjp(N("concat", {"lo": [1, 0], "hi": [4, 4]}, []), [a, b], dy)
    assert np.array_equal(da[:, 1:4], dy[:, :3]) and not da[:, :1].any() and not da[:, 4:].any()
    assert np.array_equal(db[:, :4], dy[:, 3:]) and not db[:, 4:].any()
    # global average pool spreads the gradient evenly; a fully connected layer is a matrix product
    (dg,), _ = node_vjp(N("global_avgpool", {}, []), [xs[0]], dy[:, :, :1, :1])
    assert np.allclose(dg, np.broadcast_to(dy[:, :, :1, :1] / 12.0, dg.shape))
    wfc, bfc = rng.standard_normal((5, 7)), rng.standard_normal(5)
    x1, d1 = rng.standard_normal((3, 7, 1, 1)), rng.standard_normal((3, 5, 1, 1))
    (dx,), (dw, dbias) = node_vjp(N("fc", {}, [wfc, bfc]), [x1], d1)
    assert np.allclose(dx[:, :, 0, 0], d1[:, :, 0, 0] @ wfc) and np.allclose(dw, d1[:, :, 0, 0].T @ x1[:, :, 0, 0])
    assert np.allclose(dbias, d1.sum(axis=(0, 2, 3)))
    # a tie in a max pool goes to one tap only (the first in window order): the gradient is not duplicated
    (dx,), _ = node_vjp(N("pool", {"mode": "max", "stride": 1, "pad": 1}, []), [np.ones((1, 1, 3, 3))], np.ones((1, 1, 3, 3)))
    assert dx.sum() == 9.0
    # one step of gradient descent on L = <w, g> lowers L by lr * |g|^2
    w0 = [rng.standard_normal((4, 3)).astype(np.float32)]
    g0 = [rng.standard_normal((4, 3))]
    w1 = sgd_step(w0, g0, 0.01)
    assert w1[0].dtype == np.float32
    assert np.isclose(float((w0[0] * g0[0]).sum() - (w1[0] * g0[0]).sum()), 0.01 * float((g0[0] ** 2).sum()), rtol=1e-4)
