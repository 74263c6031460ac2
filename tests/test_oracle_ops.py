"""Pins for the oracle's operator formulas: index-by-index brute force on tiny
inputs, closed forms, and torch.nn.functional on CPU as a library special case."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads
from oracle import ops
from oracle.forward import forward

R = np.random.default_rng(0)


def rnd(*shape):
    return R.standard_normal(shape).astype(np.float32)


def t64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def close(a, b, tol=2e-6):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape
    assert np.abs(a - b).max() <= tol * max(1.0, np.abs(b).max())


# ---- brute force straight from the index formulas ---------------------------
def conv_loops(x, w, stride, pad):
    n, c, h, wd = x.shape
    o, _, k, _ = w.shape
    ho, wo = (h + 2 * pad - k) // stride + 1, (wd + 2 * pad - k) // stride + 1
    y = np.zeros((n, o, ho, wo))
    for b in range(n):
        for oc in range(o):
            for i in range(ho):
                for j in range(wo):
                    acc = 0.0
                    for ic in range(c):
                        for a in range(k):
                            for bb in range(k):
                                r, s = i * stride + a - pad, j * stride + bb - pad
                                if 0 <= r < h and 0 <= s < wd:
                                    acc += float(w[oc, ic, a, bb]) * float(x[b, ic, r, s])
                    y[b, oc, i, j] = acc
    return y


def pool_loops(x, mode, stride, pad):
    n, c, h, wd = x.shape
    ho, wo = (h + 2 * pad - 3) // stride + 1, (wd + 2 * pad - 3) // stride + 1
    y = np.zeros((n, c, ho, wo))
    for b in range(n):
        for ch in range(c):
            for i in range(ho):
                for j in range(wo):
                    vals = [float(x[b, ch, i * stride + a - pad, j * stride + bb - pad])
                            for a in range(3) for bb in range(3)
                            if 0 <= i * stride + a - pad < h and 0 <= j * stride + bb - pad < wd]
                    y[b, ch, i, j] = max(vals) if mode == "max" else sum(vals) / len(vals)
    return y


@pytest.mark.parametrize("stride,pad,h,w", [(1, 1, 5, 6), (2, 1, 7, 6), (1, 0, 5, 5), (2, 0, 8, 7)])
def test_conv3x3_brute_force(stride, pad, h, w):
    x, k = rnd(2, 3, h, w), rnd(4, 3, 3, 3)
    close(ops.conv3x3(x, k, stride, pad), conv_loops(x, k, stride, pad))


@pytest.mark.parametrize("k,stride", [(3, 1), (3, 2), (5, 1), (5, 2)])
def test_dwconv_brute_force(k, stride):
    x, w = rnd(2, 3, 7, 6), rnd(3, k, k)
    dense = np.zeros((3, 3, k, k), np.float32)
    for c in range(3):
        dense[c, c] = w[c]                      # depthwise = dense conv with a diagonal kernel
    close(ops.dwconv(x, w, stride), conv_loops(x, dense, stride, k // 2))


@pytest.mark.parametrize("mode", ["max", "avg"])
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (2, 0), (1, 0)])
def test_pool_brute_force(mode, stride, pad):
    x = rnd(2, 3, 7, 8)
    close(ops.pool3x3(x, mode, stride, pad), pool_loops(x, mode, stride, pad))


# ---- closed forms -------------------------------------------------------------
def test_conv1x1_is_a_matrix_product():
    x, w = rnd(2, 5, 4, 3), rnd(7, 5)
    ref = np.einsum("oc,nchw->nohw", w.astype(np.float64), x.astype(np.float64))
    close(ops.conv1x1(x, w), ref)


def test_dwconv_one_hot_kernel_is_a_shift():
    x = rnd(1, 2, 6, 6)
    w = np.zeros((2, 3, 3), np.float32)
    w[:, 1, 2] = 1.0                            # tap (row 0, col +1): y[i, j] = x[i, j + 1]
    y = ops.dwconv(x, w, 1)
    assert np.array_equal(y[..., :, :-1], x[..., :, 1:])
    assert np.all(y[..., :, -1] == 0)


def test_bn_identity_statistics_closed_form():
    x = rnd(2, 4, 3, 3)
    one, zero = np.ones(4, np.float32), np.zeros(4, np.float32)
    close(ops.bn_act(x, one, zero, zero, one, 1e-5, False), x.astype(np.float64) / np.sqrt(1 + 1e-5), 1e-7)
    y = ops.bn_act(x, one, zero, zero, one, 1e-5, True)
    assert (y >= 0).all() and np.array_equal(y > 0, x > 0)


def test_bn_affine_per_channel():
    x = rnd(1, 3, 2, 2)
    g, b, m, v = rnd(3), rnd(3), rnd(3), np.abs(rnd(3)) + 0.5
    y = ops.bn_act(x, g, b, m, v, 1e-3, False)
    for c in range(3):
        ref = float(g[c]) * (x[0, c].astype(np.float64) - float(m[c])) / np.sqrt(float(v[c]) + 1e-3) + float(b[c])
        close(y[0, c], ref)


def test_avg_pool_of_a_constant_and_max_pool_of_a_ramp():
    x = np.full((1, 2, 6, 6), 3.25, np.float32)
    for stride, pad in [(1, 1), (2, 1), (2, 0)]:
        assert np.all(ops.pool3x3(x, "avg", stride, pad) == 3.25)   # divisor counts in-bounds taps only
    ramp = np.arange(36, dtype=np.float32).reshape(1, 1, 6, 6)
    y = ops.pool3x3(ramp, "max", 1, 1)
    ii, jj = np.minimum(np.arange(6) + 1, 5), np.minimum(np.arange(6) + 1, 5)
    assert np.array_equal(y[0, 0], ramp[0, 0][np.ix_(ii, jj)])       # bottom-right in-bounds neighbour


def test_add_concat_gap_fc_closed_forms():
    a, b, c = rnd(1, 4, 3, 3), rnd(1, 4, 3, 3), rnd(1, 4, 3, 3)
    close(ops.add_n([a, b, c]), a.astype(np.float64) + b + c)
    y = ops.concat([a, b], [1, 0], [3, 4])
    assert y.shape == (1, 6, 3, 3) and np.array_equal(y[:, :2], a[:, 1:3]) and np.array_equal(y[:, 2:], b)
    close(ops.global_avgpool(a), a.astype(np.float64).sum(axis=(2, 3), keepdims=True) / 9)
    x, w, bias = rnd(3, 5, 1, 1), rnd(2, 5), rnd(2)
    close(ops.fc(x, np.zeros_like(w), bias)[:, :, 0, 0], np.tile(bias, (3, 1)))
    close(ops.fc(x, w, bias)[:, :, 0, 0], x[:, :, 0, 0].astype(np.float64) @ w.T.astype(np.float64) + bias)


# ---- library special case: torch on CPU in fp64 --------------------------------
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0), (2, 0)])
def test_against_torch_conv_and_pool(stride, pad):
    x, w = rnd(2, 6, 11, 9), rnd(5, 6, 3, 3)
    close(ops.conv3x3(x, w, stride, pad), F.conv2d(t64(x), t64(w), stride=stride, padding=pad).numpy())
    close(ops.pool3x3(x, "max", stride, pad), F.max_pool2d(t64(x), 3, stride, pad).numpy())
    close(ops.pool3x3(x, "avg", stride, pad),
          F.avg_pool2d(t64(x), 3, stride, pad, count_include_pad=False).numpy())


def test_against_torch_depthwise_bn_linear():
    x = rnd(2, 6, 9, 10)
    for k in (3, 5):
        for stride in (1, 2):
            w = rnd(6, k, k)
            ref = F.conv2d(t64(x), t64(w)[:, None], stride=stride, padding=k // 2, groups=6).numpy()
            close(ops.dwconv(x, w, stride), ref)
    g, b, m, v = rnd(6), rnd(6), rnd(6), np.abs(rnd(6)) + 0.1
    ref = F.batch_norm(t64(x), t64(m), t64(v), t64(g), t64(b), False, 0.0, 1e-5).numpy()
    close(ops.bn_act(x, g, b, m, v, 1e-5, False), ref)
    close(ops.bn_act(x, g, b, m, v, 1e-5, True), np.maximum(ref, 0))
    xv, w, bias = rnd(3, 8, 1, 1), rnd(4, 8), rnd(4)
    close(ops.fc(xv, w, bias)[:, :, 0, 0], F.linear(t64(xv)[:, :, 0, 0], t64(w), t64(bias)).numpy())


# ---- whole DAG ------------------------------------------------------------------
def test_forward_tiny_cell_against_hand_composition():
    w = workloads.make("tiny_cell")
    nd = w.nodes
    x = w.input.astype(np.float64)
    a = np.einsum("oc,nchw->nohw", nd[1].weights[0].astype(np.float64), x) / np.sqrt(1 + 1e-5)
    a = np.maximum(a, 0)
    d = F.conv2d(t64(x), t64(nd[4].weights[0])[:, None], padding=1, groups=16).numpy()
    b = np.einsum("oc,nchw->nohw", nd[5].weights[0].astype(np.float64), d) / np.sqrt(1 + 1e-5)
    out = forward(w)[7]
    close(out, a + b, 1e-6)


@pytest.mark.parametrize("name", ["chain50", "random200"])
def test_forward_shapes_and_finiteness(name):
    w = workloads.make(name)
    out = forward(w, keep=range(len(w.nodes)))
    for i, nd in enumerate(w.nodes):
        assert out[i].shape == nd.shape and out[i].dtype == np.float32
        assert np.isfinite(out[i]).all()


def test_forward_all_ten_ops_against_hand_composition_with_torch():
    """A 17-node DAG that uses every operator kind, including the strided / padded / sliced /
    multi-operand variants, composed a second time by hand from torch.nn.functional in fp64.
    Pins forward.eval_node's plumbing: which weight goes where, stride and pad, pool mode,
    concat slices in predecessor order, add_n over several operands, fc with its bias."""
    from workloads.model import Builder
    b = Builder("all_ops")
    x = b.input(2, 6, 11, 9)
    c3 = b.conv3x3(x, 8, stride=2, pad=1)           # 1  -> [2, 8, 6, 5]
    bn = b.bn_act(c3, relu=True)                    # 2
    c3b = b.conv3x3(x, 8, stride=2, pad=1)          # 3
    bn2 = b.bn_act(c3b, relu=False, eps=1e-3)       # 4
    dw = b.dwconv(bn, 5, 1)                         # 5
    pw = b.conv1x1(dw, 8)                           # 6
    mx = b.pool(bn2, "max", 1, 1)                   # 7
    av = b.pool(bn2, "avg", 1, 1)                   # 8
    s3 = b.add_n([pw, mx, av])                      # 9
    r = b.relu(s3)                                  # 10
    dw2 = b.dwconv(x, 3, 2)                         # 11 -> [2, 6, 6, 5]
    cat = b.concat([r, dw2, bn2], slices=[(2, 7), (0, 6), (1, 4)])   # 12: 5 + 6 + 3 = 14 channels
    p2 = b.pool(cat, "avg", 2, 0)                   # 13 -> [2, 14, 2, 2]
    c3c = b.conv3x3(p2, 10, stride=1, pad=1)        # 14 -> [2, 10, 2, 2]
    gap = b.global_avgpool(c3c)                     # 15
    fc = b.fc(gap, 7)                               # 16
    rng = np.random.default_rng(5)
    b.draw_weights(rng, 0.3, "random")
    w = b.finish(rng, outputs=[fc, cat, s3])
    nd = w.nodes
    assert {n.op for n in nd} == set(workloads.OPS)
    out = forward(w, keep=range(len(nd)))

    def bn_t(t, node):
        g, be, m, v = (t64(a) for a in node.weights)
        y = F.batch_norm(t, m, v, g, be, False, 0.0, node.params["eps"])
        return F.relu(y) if node.params["relu"] else y

    X = t64(w.input)
    t1 = F.conv2d(X, t64(nd[1].weights[0]), stride=2, padding=1)
    t2 = bn_t(t1, nd[2])
    t3 = F.conv2d(X, t64(nd[3].weights[0]), stride=2, padding=1)
    t4 = bn_t(t3, nd[4])
    t5 = F.conv2d(t2, t64(nd[5].weights[0])[:, None], stride=1, padding=2, groups=8)
    t6 = F.conv2d(t5, t64(nd[6].weights[0])[:, :, None, None])
    t7 = F.max_pool2d(t4, 3, stride=1, padding=1)
    t8 = F.avg_pool2d(t4, 3, stride=1, padding=1, count_include_pad=False)
    t9 = t6 + t7 + t8
    t10 = F.relu(t9)
    t11 = F.conv2d(X, t64(nd[11].weights[0])[:, None], stride=2, padding=1, groups=6)
    t12 = torch.cat([t10[:, 2:7], t11[:, 0:6], t4[:, 1:4]], dim=1)
    t13 = F.avg_pool2d(t12, 3, stride=2, padding=0)
    t14 = F.conv2d(t13, t64(nd[14].weights[0]), stride=1, padding=1)
    t15 = t14.mean(dim=(2, 3), keepdim=True)
    t16 = F.linear(t15[:, :, 0, 0], t64(nd[16].weights[0]), t64(nd[16].weights[1]))[:, :, None, None]
    for v, t in {1: t1, 2: t2, 4: t4, 5: t5, 6: t6, 7: t7, 8: t8, 9: t9, 10: t10, 11: t11, 12: t12, 13: t13, 14: t14,
                 15: t15, 16: t16}.items():
        close(out[v], t.numpy(), 5e-6)       # fp32 storage of every intermediate tensor in the oracle
