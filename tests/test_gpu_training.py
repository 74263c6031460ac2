"""GPU parity of a whole training iteration (Section 5 of the paper, training results): forward pass,
backward pass and SGD update registered as ONE DAG through the C ABI, scheduled by the same
Algorithm 1 and replayed - against the CPU oracle's backward pass (oracle/backward.py).

Tolerance: per tensor, max|gpu - ref| <= 1e-4 * max|ref| (fp32 on the GPU, fp64 in the oracle).

Where a floating-point value decides a branch - which elements a ReLU passes, which tap of a max-pool
window attains the maximum - both sides must decide on the same data, or an element whose forward value
differs in the last bit around the threshold would flip. The comparison therefore runs the oracle's
operator-by-operator backward rules (oracle.backward.node_vjp, descending node id, exactly as
oracle.backward.backward does) on the forward tensors the GPU stored, which are themselves checked
against the oracle's forward pass. For a batch-norm with ReLU the mask is read off the stored forward
result (y > 0), which is what the kernel's own recomputation gives bit for bit.
"""
import numpy as np
import pytest

import workloads
from oracle.backward import backward as oracle_backward, node_vjp, sgd_step
from oracle.forward import forward
from paper_2012_02732_amd import GraphRunner, binding as B

pytestmark = pytest.mark.gpu
TOL = 1e-4
DEV = "cuda:0"


def rel_err(got, ref):
    ref64 = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64).reshape(ref64.shape) - ref64).max() / max(np.abs(ref64).max(), 1e-30))


def oracle_backward_on(fwd, values, seeds):
    """oracle.backward.backward with the forward values given (fp32 tensors per node) instead of recomputed."""
    n = len(fwd.nodes)
    d_value = {v: np.zeros(values[v].shape) for v in range(n)}
    d_weight = {}
    for o, s in seeds.items():
        d_value[o] = d_value[o] + np.asarray(s, dtype=np.float64)
    for v in range(n - 1, -1, -1):
        nd = fwd.nodes[v]
        if nd.op == "input":
            continue
        ins = [values[u] for u in nd.preds]
        dy = d_value[v]
        if nd.op == "bn_act" and nd.params["relu"]:
            # the ReLU's decision, taken on the stored forward result; the affine part by the oracle's rule
            dy = dy * (values[v] > 0)
            plain = type(nd)(nd.op, nd.preds, dict(nd.params, relu=0), nd.weights, nd.shape)
            dins, dws = node_vjp(plain, ins, dy)
        else:
            dins, dws = node_vjp(nd, ins, dy)
        for u, d in zip(nd.preds, dins):
            d_value[u] = d_value[u] + d
        d_weight[v] = dws
    return d_value, d_weight


def run_training_step(tw, mode, plan_trials=1):
    """One replay of the training DAG from the initial weights: (forward + gradient tensors, new weights)."""
    r = GraphRunner(tw, DEV)
    r.prepare(plan_trials=plan_trials)
    try:
        fwd = tw.forward
        for v, nd in enumerate(fwd.nodes):                       # capture must have left the weights alone
            for j, w in enumerate(nd.weights):
                assert np.array_equal(r.weight(v, j), w), ("weights changed during capture", v, j)
        r.arena.zero_()
        for node_id, value in tw.inputs.items():
            r.set_input(value, node_id)
        r.replay(mode)
        r.sync()
        tensors = {v: r.output(v) for v in range(len(tw.nodes))}
        new_w = {(v, j): r.weight(v, j) for (v, j) in tw.update_of}
        return tensors, new_w
    finally:
        r.close()


def check_training(fwd, seeds, lr, modes, end_to_end):
    tw = workloads.training_graph(fwd, lr, seeds)
    ref_fwd = forward(fwd, keep=range(len(fwd.nodes)))
    first = None
    for mode in modes:
        tensors, new_w = run_training_step(tw, mode)
        worst = 0.0
        # 1. the forward pass inside the training DAG (the GEMM kernels that read weights in place)
        for v in range(1, len(fwd.nodes)):
            e = rel_err(tensors[v], ref_fwd[v])
            assert e <= TOL, ("forward", mode, v, fwd.nodes[v].op, e)
            worst = max(worst, e)
        # 2. every gradient against the oracle's backward rules on those forward values
        values = {v: tensors[v] for v in range(len(fwd.nodes))}
        d_value, d_weight = oracle_backward_on(fwd, values, seeds)
        for v, node in tw.grad_of.items():
            e = rel_err(tensors[node], d_value[v])
            assert e <= TOL, ("dL/dvalue", mode, v, fwd.nodes[v].op, e)
            worst = max(worst, e)
        for (v, j), (node, off, numel) in tw.wgrad_of.items():
            got = tensors[node].reshape(-1)[off:off + numel]
            e = rel_err(got, np.asarray(d_weight[v][j]).reshape(-1))
            assert e <= TOL, ("dL/dweight", mode, v, j, fwd.nodes[v].op, e)
            worst = max(worst, e)
        # 3. the update, in place in the caller's weight buffers
        for (v, j) in tw.update_of:
            want = sgd_step([fwd.nodes[v].weights[j]], [d_weight[v][j].reshape(fwd.nodes[v].weights[j].shape)], lr)[0]
            e = rel_err(new_w[(v, j)], want)
            assert e <= TOL, ("sgd", mode, v, j, e)
        for v, nd in enumerate(fwd.nodes):                       # batch-norm statistics stay as they were
            if nd.op == "bn_act":
                assert (v, 2) not in tw.update_of and (v, 3) not in tw.update_of
        if end_to_end:
            # 4. and the oracle's own end-to-end backward pass (its own forward values, its own decisions)
            dv, dw = oracle_backward(fwd, seeds)
            for (v, j), (node, off, numel) in tw.wgrad_of.items():
                e = rel_err(tensors[node].reshape(-1)[off:off + numel], np.asarray(dw[v][j]).reshape(-1))
                assert e <= TOL, ("end to end dL/dweight", mode, v, j, e)
        print(f"{tw.name} mode {mode}: {len(tw.nodes)} nodes, worst rel err {worst:.2e}", flush=True)
        if first is None:
            first = (tensors, new_w)
        else:                                                    # same kernels, other order: bit for bit
            for v in range(1, len(tw.nodes)):
                if tw.nodes[v].op != "input":
                    assert np.array_equal(tensors[v], first[0][v]), ("modes differ", v, tw.nodes[v].op)
            for k in new_w:
                assert np.array_equal(new_w[k], first[1][k]), ("modes differ in the update", k)


def test_training_step_tiny_cell():
    fwd = workloads.make("tiny_cell")
    rng = np.random.default_rng(1)
    out = fwd.outputs[0]
    seeds = {out: rng.standard_normal(fwd.nodes[out].shape).astype(np.float32)}
    check_training(fwd, seeds, 0.05, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT, B.NG_MODE_GRAPH_MULTI), end_to_end=True)


def test_training_step_all_operators_small():
    """Every backward operator on ragged shapes: strided and padded 3x3 convolutions, both depthwise sizes
    and strides, both pools with and without padding, sliced concat, a tensor with three readers,
    batch-norm with and without ReLU, fc with bias."""
    from workloads.model import Builder
    b = Builder("all_backward_ops")
    x = b.input(3, 5, 13, 11)
    c3 = b.bn_act(b.conv3x3(x, 12, 2, 1), relu=True)                 # [3, 12, 7, 6]
    c3b = b.bn_act(b.conv3x3(c3, 9, 1, 0), relu=False)               # [3, 9, 5, 4]
    d5 = b.dwconv(c3, 5, 2)                                          # [3, 12, 4, 3]
    d3 = b.dwconv(c3, 3, 1)
    pw = b.conv1x1(d3, 12)
    mx = b.pool(c3, "max", 1, 1)
    av = b.pool(pw, "avg", 1, 1)
    s3 = b.add_n([pw, mx, av])
    r = b.relu(s3)
    mx2 = b.pool(r, "max", 2, 0)                                     # [3, 12, 3, 2]
    av2 = b.pool(r, "avg", 2, 1)                                     # [3, 12, 4, 3]
    cat = b.concat([d5, av2], slices=[(2, 9), (0, 12)])              # 19 channels
    g1 = b.global_avgpool(b.conv3x3(cat, 8, 1, 1))
    g2 = b.global_avgpool(b.conv1x1(mx2, 8))
    g3 = b.global_avgpool(b.conv1x1(c3b, 8))
    f = b.fc(b.add_n([g1, g2, g3]), 6)
    rng = np.random.default_rng(2)
    b.draw_weights(rng, 0.3, "random")
    fwd = b.finish(rng, outputs=[f])
    seeds = {f: rng.standard_normal(fwd.nodes[f].shape).astype(np.float32)}
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT), end_to_end=False)


@pytest.mark.parametrize("shape,kernel", [((2, 5, 40, 36), "pool3x3_dgrad"), ((3, 7, 9, 10), "pool3x3_dgrad_lds"),
                                          ((2, 3, 32, 32), "pool3x3_dgrad_lds"), ((5, 3, 16, 16), "pool3x3_dgrad_lds")])
def test_training_pool_backward_plane_sizes(shape, kernel):
    """Pool backward through both of its kernels: planes a workgroup stages whole in LDS (up to 1024 pixels; several
    small planes per workgroup with a ragged last group) and larger ones; maximum and average, strides 1 and 2,
    with and without padding. Ties are frequent: the inputs of the pools are rounded to a few values."""
    from workloads.model import Builder
    b = Builder("pool_backward")
    x = b.input(*shape)
    pw = b.conv1x1(x, shape[1])
    outs = []
    for mode, stride, pad in (("max", 1, 1), ("avg", 1, 1), ("max", 2, 0), ("avg", 2, 1), ("max", 2, 1)):
        outs.append(b.global_avgpool(b.pool(pw, mode, stride, pad)))
    f = b.fc(b.add_n(outs), 4)
    rng = np.random.default_rng(5)
    b.draw_weights(rng, 0.3, "random")
    fwd = b.finish(rng, outputs=[f])
    fwd.input = (np.round(fwd.input * 2.0) / 2.0).astype(np.float32)
    for nd in fwd.nodes:                                             # conv1x1 of coarse values with coarse weights: many equal taps
        if nd.op == "conv1x1":
            nd.weights[0] = (np.round(nd.weights[0] * 4.0) / 4.0).astype(np.float32)
    seeds = {f: rng.standard_normal(fwd.nodes[f].shape).astype(np.float32)}
    tw = workloads.training_graph(fwd, 0.01, seeds)
    r = GraphRunner(tw)
    r.schedule()
    r.plan()
    names = {B.ng_planned_task_kernel(r.g, v) for v, nd in enumerate(tw.nodes) if nd.op == "pool_dgrad"}
    r.close()
    assert names == {kernel}, names
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT), end_to_end=False)


@pytest.mark.parametrize("shape,cout,kernel", [((2, 3, 16, 16), 7, "conv3x3_wgrad_px_16"), ((3, 5, 8, 32), 44, "conv3x3_wgrad_px_16"),
                                               ((1, 20, 16, 48), 40, "conv3x3_wgrad_px_32"), ((2, 3, 12, 20), 9, "gemm_conv3x3_wgrad")])
def test_training_conv3x3_weight_gradient_kernels(shape, cout, kernel):
    """conv3x3 weight gradient, stride 1 and padding 1: rows of a multiple of 16 pixels read the shifted input planes
    128 bits at a time (both block sizes, row ends, first and last row, ragged channel counts); other widths take the
    gather GEMM."""
    from workloads.model import Builder
    b = Builder("conv3x3_wgrad")
    x = b.input(*shape)
    c = b.bn_act(b.conv3x3(x, cout, 1, 1), relu=True)
    f = b.fc(b.global_avgpool(c), 5)
    rng = np.random.default_rng(6)
    b.draw_weights(rng, 0.3, "random")
    fwd = b.finish(rng, outputs=[f])
    seeds = {f: rng.standard_normal(fwd.nodes[f].shape).astype(np.float32)}
    tw = workloads.training_graph(fwd, 0.01, seeds)
    r = GraphRunner(tw)
    r.schedule()
    r.plan()
    names = {B.ng_planned_task_kernel(r.g, v) for v, nd in enumerate(tw.nodes) if nd.op == "conv3x3_wgrad"}
    r.close()
    assert names == {kernel}, names
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT), end_to_end=False)


@pytest.mark.parametrize("shape,kernel", [((2, 5, 8, 8), "dwconv_dgrad_lds"), ((3, 7, 16, 16), "dwconv_dgrad_lds"),
                                          ((1, 3, 32, 32), "dwconv_dgrad_lds"), ((2, 4, 10, 14), "dwconv_dgrad"), ((1, 2, 40, 36), "dwconv_dgrad")])
def test_training_depthwise_backward_kernels(shape, kernel):
    """Depthwise backward, both filter sizes and strides in one graph: planes of up to 1024 pixels with rows of a multiple
    of four go through LDS (several small planes per workgroup, a ragged last group), the others through the
    element-wise kernel; the weight gradient likewise has its LDS path and its general one."""
    from workloads.model import Builder
    b = Builder("depthwise_backward")
    x = b.input(*shape)
    pw = b.conv1x1(x, shape[1])
    outs = [b.global_avgpool(b.dwconv(pw, k, s)) for k in (3, 5) for s in (1, 2)]
    f = b.fc(b.add_n(outs), 4)
    rng = np.random.default_rng(7)
    b.draw_weights(rng, 0.3, "random")
    fwd = b.finish(rng, outputs=[f])
    seeds = {f: rng.standard_normal(fwd.nodes[f].shape).astype(np.float32)}
    tw = workloads.training_graph(fwd, 0.01, seeds)
    r = GraphRunner(tw)
    r.schedule()
    r.plan()
    names = {B.ng_planned_task_kernel(r.g, v) for v, nd in enumerate(tw.nodes) if nd.op == "dwconv_dgrad"}
    r.close()
    assert names == {kernel}, names
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT), end_to_end=False)


@pytest.mark.parametrize("shape,cout", [((3, 20, 6, 6), 24), ((2, 20, 8, 8), 24), ((5, 12, 4, 4), 40), ((1, 36, 16, 16), 7), ((2, 8, 5, 4), 150)])
def test_training_conv1x1_pixel_kernels(shape, cout):
    """conv1x1 forward, input gradient and weight gradient through the kernels that read pixels 128 bits at a time:
    ragged last pixel groups, row fragments beyond Cout, K that ends inside a slice of 16 channels, a K range of the
    weight gradient that ends inside a split, the batch-norm applied by the forward kernel (with and without ReLU),
    and two convolutions in a row so that both gradients of the first are needed."""
    from workloads.model import Builder
    b = Builder("conv1x1_pixels")
    x = b.input(*shape)
    c1 = b.bn_act(b.conv1x1(x, cout), relu=True)
    c2 = b.bn_act(b.conv1x1(c1, shape[1]), relu=False)
    f = b.fc(b.global_avgpool(b.add_n([c2, x])), 3)
    rng = np.random.default_rng(8)
    b.draw_weights(rng, 0.3, "random")
    fwd = b.finish(rng, outputs=[f])
    seeds = {f: rng.standard_normal(fwd.nodes[f].shape).astype(np.float32)}
    tw = workloads.training_graph(fwd, 0.01, seeds)
    r = GraphRunner(tw)
    r.schedule()
    r.plan()
    names = {nd.op: set() for nd in tw.nodes}
    for v, nd in enumerate(tw.nodes):
        names[nd.op].add(B.ng_planned_task_kernel(r.g, v))
    r.close()
    hw = shape[2] * shape[3]
    assert "conv1x1_px_fwd" in names["conv1x1"] and "conv1x1_px_dgrad" in names["conv1x1_dgrad"], names   # (a K that is no multiple of 4: gather GEMM forward)
    assert (hw % 16 != 0) == ("gemm_conv1x1_wgrad" in names["conv1x1_wgrad"]), names
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT, B.NG_MODE_GRAPH_MULTI), end_to_end=False)


def test_training_step_nas_cell_batch32_cifar():
    """The paper's training setting: batch 32, 32 x 32 inputs. One normal and one reduction cell of the
    NASNet-style recipe between a 3x3 stem and a 10-way classifier; 259 tasks in one DAG."""
    fwd = workloads.nas_cell_cifar()
    rng = np.random.default_rng(3)
    out = fwd.outputs[0]
    seeds = {out: (rng.standard_normal(fwd.nodes[out].shape) / 32.0).astype(np.float32)}
    check_training(fwd, seeds, 0.01, (B.NG_MODE_GRAPH_SINGLE, B.NG_MODE_DEVICE_RESIDENT), end_to_end=False)


def test_training_replays_keep_training():
    """Each replay is one more SGD step on the caller's weights: two replays equal two oracle steps."""
    fwd = workloads.make("tiny_cell")
    rng = np.random.default_rng(4)
    out = fwd.outputs[0]
    seeds = {out: rng.standard_normal(fwd.nodes[out].shape).astype(np.float32)}
    lr = 0.05
    tw = workloads.training_graph(fwd, lr, seeds)
    r = GraphRunner(tw, DEV)
    r.prepare()
    try:
        for node_id, value in tw.inputs.items():
            r.set_input(value, node_id)
        for _ in range(2):
            r.replay(B.NG_MODE_AUTO)
            r.sync()
        got = {k: r.weight(*k) for k in tw.update_of}
    finally:
        r.close()
    import copy
    cur = copy.deepcopy(fwd)
    for _ in range(2):
        _, dw = oracle_backward(cur, seeds)
        for (v, j) in tw.update_of:
            cur.nodes[v].weights[j] = sgd_step([cur.nodes[v].weights[j]], [dw[v][j].reshape(cur.nodes[v].weights[j].shape)], lr)[0]
    for (v, j) in tw.update_of:
        assert rel_err(got[(v, j)], cur.nodes[v].weights[j]) <= TOL, (v, j)
