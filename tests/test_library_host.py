"""Host-only tests of the C-ABI library: it loads without a GPU, exports every declared
symbol, infers shapes, and its scheduling pass matches the oracle bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads
from workloads.model import Builder, Node, Workload
from oracle.schedule import schedule as oracle_schedule, schedule_exact as oracle_schedule_exact
from oracle import checks
from oracle.memory import plan_is_safe as memory_plan_is_safe
from paper_2012_02732_amd import GraphRunner, binding as B
from dag_util import random_dag, layered_dag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def abstract_workload(n, edges):
    """A DAG with no tensor meaning: sources are inputs, one predecessor -> relu, several -> add_n."""
    preds = [[] for _ in range(n)]
    for u, v in sorted(set(edges)):
        preds[v].append(u)
    nodes = []
    for v in range(n):
        if not preds[v]:
            nodes.append(Node("input", [], dict(n=1, c=2, h=2, w=2), [], (1, 2, 2, 2)))
        elif len(preds[v]) == 1:
            nodes.append(Node("relu", preds[v], {}, [], (1, 2, 2, 2)))
        else:
            nodes.append(Node("add_n", preds[v], {}, [], (1, 2, 2, 2)))
    return Workload("abstract", nodes, np.zeros((1, 2, 2, 2), np.float32), [n - 1])


def assert_same_schedule(lib_sched, scaffold, o):
    assert lib_sched["meg"] == o.meg
    assert lib_sched["n_matching"] == len(o.matching)
    assert lib_sched["chain_of"] == o.chain_of and lib_sched["n_chains"] == o.n_chains
    assert lib_sched["stream_of"] == o.stream_of and lib_sched["n_streams"] == o.n_streams
    assert lib_sched["sync"] == o.sync
    assert lib_sched["event_of"] == o.event_of and lib_sched["n_events"] == o.n_events
    assert lib_sched["order"] == o.order
    assert scaffold == (o.fork, o.join)


def test_header_symbols_are_exported():
    header = open(os.path.join(ROOT, "include", "nimble_graph.h")).read()
    declared = set(re.findall(r"\b(ng_[a-z_]+)\s*\(", header))
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    for name in declared:
        assert hasattr(B.lib, name), name
    assert "gfx950" in B.ng_version()


def test_schedule_parity_on_random_tiny_dags():
    rng = np.random.default_rng(123)
    for i in range(3000):
        n = int(rng.integers(1, 17))
        e = random_dag(rng, n, float(rng.uniform(0.1, 0.7)))
        r = GraphRunner(abstract_workload(n, e))
        s = r.schedule()
        assert_same_schedule(s, B.ng_get_scaffold(r.g), oracle_schedule(n, e))
        r.close()


def test_schedule_parity_on_medium_dags():
    rng = np.random.default_rng(7)
    for _ in range(60):
        n, e = layered_dag(rng, int(rng.integers(3, 15)), 9)
        r = GraphRunner(abstract_workload(n, e))
        assert_same_schedule(r.schedule(), B.ng_get_scaffold(r.g), oracle_schedule(n, e))
        r.close()
    for _ in range(20):
        n = int(rng.integers(40, 160))
        e = random_dag(rng, n, float(rng.uniform(0.01, 0.08)))
        r = GraphRunner(abstract_workload(n, e))
        assert_same_schedule(r.schedule(), B.ng_get_scaffold(r.g), oracle_schedule(n, e))
        r.close()


def check_exact_schedule(n, e, lib_sched, scaffold):
    """The library's exact assignment against the oracle's: several partitions can be optimal, so
    what is unique is compared (E', Algorithm 1's chains, stream and synchronisation counts) and
    the rest is checked for validity (streams are chains of the closure, labelled in order of
    their first node; Lambda = the cross-stream E' edges; events and scaffolding consistent)."""
    o = oracle_schedule_exact(n, e)
    assert lib_sched["meg"] == o.meg and lib_sched["n_matching"] == len(o.matching)
    assert lib_sched["chain_of"] == o.chain_of and lib_sched["n_chains"] == o.n_chains
    assert lib_sched["n_streams"] == o.n_streams and len(lib_sched["sync"]) == len(o.sync)
    f = lib_sched["stream_of"]
    assert checks.has_max_logical_concurrency(n, e, f)
    firsts = [f.index(st) for st in range(lib_sched["n_streams"])]
    assert firsts == sorted(firsts) and f[0] == 0 and sorted(set(f)) == list(range(lib_sched["n_streams"]))
    assert lib_sched["sync"] == [(u, v) for u, v in o.meg if f[u] != f[v]]
    producers = sorted({u for u, _ in lib_sched["sync"]})
    assert [lib_sched["event_of"][u] for u in producers] == list(range(len(producers)))
    assert lib_sched["n_events"] == len(producers) and all((ev >= 0) == (u in producers) for u, ev in enumerate(lib_sched["event_of"]))
    if n <= 16:                                   # path enumeration: tiny DAGs only
        assert checks.plan_is_safe(n, e, f, lib_sched["sync"])
    waits = {v for _, v in lib_sched["sync"]}
    first_of = {st: f.index(st) for st in range(lib_sched["n_streams"])}
    assert scaffold == (sorted(st for st, v in first_of.items() if st != 0 and v not in waits),
                        sorted(st for st in first_of if st != 0))


def test_exact_assignment_on_random_tiny_dags_and_the_known_suboptimal_case():
    rng = np.random.default_rng(321)
    cases = [(12, [(0, 1), (0, 9), (1, 2), (1, 9), (2, 4), (3, 4), (3, 5), (3, 10), (3, 11), (4, 5), (5, 6),
                   (5, 11), (7, 9), (7, 11), (8, 10)])]
    for _ in range(1500):
        n = int(rng.integers(1, 17))
        cases.append((n, random_dag(rng, n, float(rng.uniform(0.1, 0.7)))))
    for n, e in cases:
        r = GraphRunner(abstract_workload(n, e))
        B.ng_set_assignment(r.g, B.NG_ASSIGN_EXACT)
        s = r.schedule()
        check_exact_schedule(n, e, s, B.ng_get_scaffold(r.g))
        r.close()
    r = GraphRunner(abstract_workload(*cases[0]))           # the default procedure on the first case: one more
    assert len(r.schedule()["sync"]) == 6
    r.close()


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_exact_assignment_on_benchmark_configs(name):
    w = workloads.make(name)
    r = GraphRunner(w)
    B.ng_set_assignment(r.g, B.NG_ASSIGN_EXACT)
    s = r.schedule()
    check_exact_schedule(len(w.nodes), w.edges, s, B.ng_get_scaffold(r.g))
    with pytest.raises(B.NgError) as err:
        B.ng_set_assignment(r.g, B.NG_ASSIGN_ALGORITHM1)    # too late
    assert err.value.code == B.NG_ESTATE
    r.close()
    r = GraphRunner(w)
    with pytest.raises(B.NgError) as err:
        B.ng_set_assignment(r.g, 7)
    assert err.value.code == B.NG_EINVAL
    r.close()


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_configs_shapes_schedule_and_plan(name):
    w = workloads.make(name)
    r = GraphRunner(w)
    for i, nd in enumerate(w.nodes):
        assert B.ng_node_shape(r.g, i) == nd.shape
    s = r.schedule()
    assert_same_schedule(s, B.ng_get_scaffold(r.g), oracle_schedule(len(w.nodes), w.edges))
    total = r.plan()
    off, nbytes = B.ng_get_offsets(r.g)
    assert nbytes == [4 * int(np.prod(nd.shape)) for nd in w.nodes]
    # A tensor that exactly one concat takes whole, at batch 1, may live inside that concat's buffer,
    # at the byte offset of its channel block; every other buffer is private: aligned, disjoint.
    inside = {}
    for c, nd in enumerate(w.nodes):
        if nd.op != "concat" or nd.shape[0] != 1:
            continue
        first = 0
        for p, lo, hi in zip(nd.preds, nd.params["lo"], nd.params["hi"]):
            at = off[c] + 4 * first * nd.shape[2] * nd.shape[3]
            if off[p] == at and p not in inside:
                assert (lo, hi) == (0, w.nodes[p].shape[1]) and nd.preds.count(p) == 1 and w.nodes[p].op != "input"
                assert at % 16 == 0
                inside[p] = c
            first += hi - lo
    spans = sorted((off[v], nbytes[v]) for v in range(len(w.nodes)) if v not in inside)
    for (o1, b1), (o2, _) in zip(spans, spans[1:]):
        assert o1 % 256 == 0 and o1 + b1 <= o2              # aligned, disjoint: no buffer reuse
    assert spans[-1][0] + spans[-1][1] <= total
    if name == "nasnet_style":                              # the three block outputs of every cell feed the cell's concat only
        assert len(inside) == 3 * sum(nd.op == "concat" for nd in w.nodes)
    if name == "inception_style" and w.nodes[0].shape[0] > 1:
        assert not inside
    r.close()


def _in_place(w, off):
    """Pairs (tensor, concat) the plan nests on purpose: the tensor sits at its channel block."""
    pairs = set()
    for c, nd in enumerate(w.nodes):
        if nd.op != "concat":
            continue
        first = 0
        for p, lo, hi in zip(nd.preds, nd.params["lo"], nd.params["hi"]):
            if off[p] == off[c] + 4 * first * nd.shape[2] * nd.shape[3] and (lo, hi) == (0, w.nodes[p].shape[1]):
                pairs.add((p, c))
            first += hi - lo
    return pairs


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_memory_reuse_plan_is_safe_on_any_number_of_streams(name):
    """With reuse switched on the arena shrinks, and the oracle's reachability check passes: two
    tensors share bytes only if everything that touches the one is an ancestor of the producer of
    the other (or they are a concat and an input produced in place inside it)."""
    w = workloads.make(name)
    n = len(w.nodes)
    r = GraphRunner(w); r.schedule(); private = r.plan(); r.close()
    r = GraphRunner(w)
    B.ng_set_memory_reuse(r.g, True)
    r.schedule()
    total = r.plan()
    off, nbytes = B.ng_get_offsets(r.g)
    assert nbytes == [4 * int(np.prod(nd.shape)) for nd in w.nodes]
    assert all(o % 16 == 0 and o + b <= total for o, b in zip(off, nbytes))
    nested = _in_place(w, off)
    closure = set(nested)
    for a, c in list(nested):                     # nesting is transitive (a concat inside a concat), and siblings never overlap
        for c2, c3 in nested:
            if c2 == c:
                closure.add((a, c3))
    keep = [0] + list(w.outputs)
    ok = memory_plan_is_safe(n, w.edges, off, nbytes, keep,
                             nested_ok=lambda a, b: (a, b) in closure or (b, a) in closure)
    assert ok
    assert total <= private
    print(f"{name}: arena {private / 1e6:.2f} MB -> {total / 1e6:.2f} MB with reuse")
    if name in ("chain50", "nasnet_style", "inception_style"):   # deep networks: most tensors die early (a 75-wide random DAG has few ancestors to inherit from)
        assert total < 0.5 * private, (total, private)
    with pytest.raises(B.NgError) as err:
        B.ng_set_memory_reuse(r.g, False)         # too late
    assert err.value.code == B.NG_ESTATE
    r.close()


def test_memory_reuse_on_random_dags():
    rng = np.random.default_rng(99)
    shrunk = 0
    for _ in range(300):
        n = int(rng.integers(2, 40))
        e = random_dag(rng, n, float(rng.uniform(0.05, 0.5)))
        w = abstract_workload(n, e)
        r = GraphRunner(w)
        B.ng_set_memory_reuse(r.g, True)
        r.schedule()
        total = r.plan()
        off, nbytes = B.ng_get_offsets(r.g)
        keep = [v for v in range(n) if not any(b == v for _, b in e)] + [n - 1]   # the inputs and the marked output
        assert memory_plan_is_safe(n, e, off, nbytes, keep)
        shrunk += total < 256 * n
        r.close()
    assert shrunk > 100


def test_batch_changes_shapes_not_schedule():
    a, b = workloads.make("inception_style", batch=1), workloads.make("inception_style", batch=32)
    ra, rb = GraphRunner(a), GraphRunner(b)
    assert ra.schedule() == rb.schedule()
    assert B.ng_node_shape(rb.g, len(b.nodes) - 1) == (32, 1000, 1, 1)
    assert rb.plan() > 30 * ra.plan() // 2


def test_critical_path_matches_plain_dp():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n, e = layered_dag(rng, 6, 5)
        w = abstract_workload(n, e)
        r = GraphRunner(w)
        t = rng.uniform(0.5, 5.0, n).astype(np.float32)
        total, path = B.ng_critical_path(r.g, list(t))
        best = np.zeros(n)
        for v in range(n):
            best[v] = t[v] + max([best[u] for u in w.nodes[v].preds], default=0.0)
        assert abs(total - best.max()) < 1e-3
        assert abs(sum(t[v] for v in path) - total) < 1e-3
        for u, v in zip(path, path[1:]):
            assert u in w.nodes[v].preds
        r.close()


def test_task_work_formulas():
    w = workloads.make("random200")
    r = GraphRunner(w)
    for v, nd in enumerate(w.nodes):
        nbytes, flops = B.ng_task_work(r.g, v)
        n, c, h, wd = nd.shape
        if nd.op == "conv1x1":
            assert flops == 2 * 64 * 64 * 784 and nbytes == 4 * (2 * 64 * 784 + 64 * 64)
        if nd.op == "dwconv":
            assert flops == 18 * 64 * 784 and nbytes == 4 * (2 * 64 * 784 + 64 * 9)
        if nd.op == "add_n":
            assert nbytes == 4 * (len(nd.preds) + 1) * 64 * 784


# ---- error paths (no exception or abort crosses the boundary) ----------------------
def _g_with_input(shape=(1, 4, 8, 8)):
    g = B.ng_create()
    B.ng_add_input(g, shape)
    return g


def _code(fn, *a):
    with pytest.raises(B.NgError) as ei:
        fn(*a)
    return ei.value.code


def test_error_codes():
    g = _g_with_input()
    p = B.ng_op_params()
    assert _code(B.ng_add_node, g, B.NG_OP_RELU, p, [5], []) == B.NG_EINVAL          # unknown predecessor
    assert _code(B.ng_add_node, g, 99, p, [0], []) == B.NG_EINVAL                   # unknown op
    assert _code(B.ng_add_node, g, B.NG_OP_RELU, p, [], []) == B.NG_EINVAL          # no predecessor
    assert _code(B.ng_add_node, g, B.NG_OP_CONV1X1, p, [0], [0]) == B.NG_EINVAL     # cout = 0
    assert _code(B.ng_add_node, g, B.NG_OP_BN_ACT, p, [0], [0]) == B.NG_EINVAL      # wrong weight count
    p.k, p.stride = 4, 1
    assert _code(B.ng_add_node, g, B.NG_OP_DWCONV, p, [0], [0]) == B.NG_EINVAL      # k not in {3,5}
    p = B.ng_op_params()
    p.cout = 3
    assert _code(B.ng_add_node, g, B.NG_OP_FC, p, [0], [0, 0]) == B.NG_ESHAPE       # fc on an 8x8 map
    small = B.ng_add_node(g, B.NG_OP_GLOBAL_AVGPOOL, B.ng_op_params(), [0], [])
    assert _code(B.ng_add_node, g, B.NG_OP_ADD_N, B.ng_op_params(), [0, small], []) == B.NG_ESHAPE
    q = B.ng_op_params()
    q.slice_lo[0], q.slice_hi[0] = 2, 9
    assert _code(B.ng_add_node, g, B.NG_OP_CONCAT, q, [0], []) == B.NG_ESHAPE       # slice past the last channel
    q = B.ng_op_params()
    q.stride, q.pad = 1, 0
    assert _code(B.ng_add_node, g, B.NG_OP_POOL, q, [small], []) == B.NG_ESHAPE     # 3x3 window on a 1x1 map
    assert _code(B.ng_mark_output, g, 77) == B.NG_EINVAL
    assert B.ng_num_nodes(g) == 2                                                   # failed calls added nothing
    # wrong call order
    assert _code(B.ng_plan_memory, g) == B.NG_ESTATE
    assert _code(B.ng_get_schedule, g) == B.NG_ESTATE
    assert _code(B.ng_capture, g) == B.NG_ESTATE
    assert _code(B.ng_replay, g) == B.NG_ESTATE
    B.ng_schedule(g)
    assert _code(B.ng_schedule, g) == B.NG_ESTATE
    assert _code(B.ng_add_node, g, B.NG_OP_RELU, B.ng_op_params(), [0], []) == B.NG_ESTATE
    assert _code(B.ng_add_input, g, (1, 1, 1, 1)) == B.NG_ESTATE
    assert _code(B.ng_bind, g, 256, 1 << 20, [0]) == B.NG_ESTATE                    # bind before plan
    B.ng_plan_memory(g)
    assert _code(B.ng_replay_mode, g, 9) == B.NG_EINVAL
    assert "ng_replay_mode" in B.ng_last_error(g)
    B.ng_destroy(g)
    B.ng_destroy(None)                                                              # allowed

    e = B.ng_create()
    assert _code(B.ng_schedule, e) == B.NG_EINVAL                                   # empty graph
    assert _code(B.ng_add_input, e, (1, 0, 2, 2)) == B.NG_ESHAPE
    B.ng_destroy(e)


def test_bind_rejects_bad_resources_without_a_gpu():
    g = _g_with_input()
    B.ng_add_node(g, B.NG_OP_RELU, B.ng_op_params(), [0], [])
    B.ng_schedule(g)
    need = B.ng_plan_memory(g)
    assert _code(B.ng_bind, g, 0, need, [0]) == B.NG_EINVAL                         # null arena
    assert _code(B.ng_bind, g, 4096 + 4, need, [0]) == B.NG_EINVAL                  # misaligned
    assert _code(B.ng_bind, g, 4096, need - 1, [0]) == B.NG_ENOMEM                  # arena too small
    assert _code(B.ng_bind, g, 4096, need, []) in (B.NG_ENOMEM, B.NG_EINVAL)        # too few streams
    buf = (C.c_char * (need + 512))()
    host = (C.addressof(buf) + 255) // 256 * 256
    assert _code(B.ng_bind, g, host, need, [0]) == B.NG_EINVAL                      # host memory is not an arena
    assert B.ng_tensor_ptr(g, 0) == 0
    B.ng_destroy(g)


def test_bind_rejects_duplicate_stream_handles():
    g = _g_with_input()
    a = B.ng_add_node(g, B.NG_OP_RELU, B.ng_op_params(), [0], [])
    b = B.ng_add_node(g, B.NG_OP_RELU, B.ng_op_params(), [0], [])
    B.ng_add_node(g, B.NG_OP_ADD_N, B.ng_op_params(), [a, b], [])
    B.ng_schedule(g)
    assert B.ng_schedule_sizes(g)["n_streams"] == 2
    need = B.ng_plan_memory(g)
    assert _code(B.ng_bind, g, 4096, need, [0x1000, 0x1000]) == B.NG_EINVAL
    assert "same handle" in B.ng_last_error(g)
    B.ng_destroy(g)


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
@pytest.mark.parametrize("n_wg,xcds", [(256, 0), (256, 1), (64, 4), (8, 8), (512, 2), (256, 5)])
def test_device_resident_plan_covers_every_tile_once(name, n_wg, xcds):
    """The per-workgroup task lists of the device-resident replay, rehearsed on the host:
    every tile of every task is assigned exactly once, lists ascend in task id (so waits
    only ever point backwards in every list: no cyclic wait), and the completion count a
    consumer expects equals the number of workgroups its producer was split over."""
    r = GraphRunner(workloads.make(name))
    r.schedule()
    r.plan()
    d = B.ng_resident_dry_plan(r.g, n_wg, xcds)
    assert d["ok"], d
    # every task has at least one list entry, except batch-norm / ReLU tasks the planner fuses into
    # the convolution that feeds them (the self-check behind d["ok"] verifies each such pair)
    n_tasks = sum(nd.op not in ("input", "bn_act", "relu") for nd in r.workload.nodes)
    assert d["n_entries"] >= n_tasks and d["expected_us"] > 0
    if xcds == 1:
        assert d["n_far_edges"] == 0
    r.close()


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_every_planner_setting_tried_at_capture_gives_a_consistent_plan(name):
    """ng_capture plans the device-resident replay under 8 settings of the planner's cost model and
    keeps the fastest plan; each of them, rehearsed on the host, covers every tile once, keeps one
    common order with parents first and has consistent completion counts - on 8 XCDs and on fewer."""
    r = GraphRunner(workloads.make(name))
    r.schedule()
    r.plan()
    base = B.ng_resident_dry_plan(r.g, 256, 0)
    assert B.ng_resident_dry_plan_setting(r.g, 0, 256, 0) == base
    expected = set()
    for setting in range(8):
        for n_wg, xcds in ((256, 0), (256, 3), (64, 8)):
            d = B.ng_resident_dry_plan_setting(r.g, setting, n_wg, xcds)
            assert d["ok"] and d["n_entries"] > 0 and d["expected_us"] > 0, (setting, n_wg, xcds, d)
            if (n_wg, xcds) == (256, 0):
                expected.add(round(d["expected_us"], 3))
    if name in ("nasnet_style", "inception_style", "random200"):
        assert len(expected) >= 4          # the settings really lead to different plans on the branchy DAGs
    for bad in (-1, 8):
        with pytest.raises(B.NgError) as e:
            B.ng_resident_dry_plan_setting(r.g, bad, 256, 0)
        assert e.value.code == B.NG_EINVAL
    r.close()


def test_device_resident_plan_argument_checks():
    r = GraphRunner(workloads.make("tiny_cell"))
    with pytest.raises(B.NgError) as e:
        B.ng_resident_dry_plan(r.g, 256, 0)
    assert e.value.code == B.NG_ESTATE
    r.schedule()
    r.plan()
    for bad in [(0, 0), (12, 0), (256, 9), (256, -1), (-8, 8)]:
        with pytest.raises(B.NgError) as e:
            B.ng_resident_dry_plan(r.g, *bad)
        assert e.value.code == B.NG_EINVAL
    # queries about the captured replay are refused before ng_capture (no GPU needed to find that out)
    for early in (B.ng_resident_fusion, B.ng_resident_sizes, B.ng_resident_xcd_mapping, B.ng_auto_mode, B.ng_resident_plan_kept):
        with pytest.raises(B.NgError) as e:
            early(r.g)
        assert e.value.code == B.NG_ESTATE, early.__name__
    # the number of planner settings ng_capture tries: 1..8
    for bad in (0, 9, -1):
        with pytest.raises(B.NgError) as e:
            B.ng_resident_plan_trials(r.g, bad)
        assert e.value.code == B.NG_EINVAL
    B.ng_resident_plan_trials(r.g, 1)
    B.ng_resident_plan_trials(r.g, 8)
    r.close()


# ---- the multi-stream HIP graph's edge list, pinned on the CPU ------------------------------

def _graph_order_is_safe(w, launched_by, graph_edges):
    """Appendix A, safe plan, applied to the graph that is really launched: for every edge (u, v)
    of E, each kernel node that writes (part of) u's tensor must reach, through graph edges, the
    kernel node that computes v. Written from the definitions: a fused batch-norm's tensor is written
    by its convolution's node, an in-place concat's tensor by the nodes of its inputs, and an in-place
    concat itself computes nothing."""
    n = len(w.nodes)

    def writers(t):
        if launched_by[t] == -1:
            return set()                                    # network input: written before the launch
        if launched_by[t] == -2:
            return set().union(*[writers(p) for p in w.nodes[t].preds])
        return {launched_by[t]}

    reach = checks.reachable(n, graph_edges)
    for u, v in w.edges:
        if launched_by[v] < 0:
            continue                                        # v runs nothing
        runner = launched_by[v]
        for k in writers(u):
            if k != runner and not reach[k][runner]:
                return False, (u, v, k, runner)
    # every graph edge points forward in the submission order (ascending id): the graph is acyclic
    return all(a < b for a, b in graph_edges), None


def _exact_and_default(w):
    for assignment in (B.NG_ASSIGN_ALGORITHM1, B.NG_ASSIGN_EXACT):
        for fuse in (True, False):
            r = GraphRunner(w)
            B.ng_set_assignment(r.g, assignment)
            sched = r.schedule()
            r.plan()
            launched_by, ge = B.ng_get_graph_edges(r.g, fuse)
            r.close()
            yield assignment, fuse, sched, launched_by, ge


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_multi_stream_graph_edges_order_every_dependency_on_the_configs(name):
    w = workloads.make(name)
    if len(w.nodes) > 300:                                   # closure by relaxation is cubic: keep the big ones to the default assignment
        runs = [(B.NG_ASSIGN_ALGORITHM1, f) for f in (True, False)]
    else:
        runs = [(a, f) for a in (B.NG_ASSIGN_ALGORITHM1, B.NG_ASSIGN_EXACT) for f in (True, False)]
    for assignment, fuse in runs:
        r = GraphRunner(w)
        B.ng_set_assignment(r.g, assignment)
        sched = r.schedule()
        r.plan()
        launched_by, ge = B.ng_get_graph_edges(r.g, fuse)
        r.close()
        ok, why = _graph_order_is_safe(w, launched_by, ge)
        assert ok, (name, assignment, fuse, why)
        ops = [nd.op for nd in w.nodes]
        if fuse:
            # what is not launched: batch-norms / ReLUs behind a convolution, concats with all inputs in place
            assert all(ops[v] in ("bn_act", "relu") and ops[launched_by[v]] in ("conv1x1", "conv3x3", "fc")
                       for v in range(len(ops)) if launched_by[v] not in (v, -1, -2))
            assert all(ops[v] == "concat" for v in range(len(ops)) if launched_by[v] == -2)
        else:
            assert all(launched_by[v] == (v if ops[v] != "input" else -1) for v in range(len(ops)))
            # one kernel per task: the edges are exactly FIFO neighbours on a stream plus Lambda
            last, fifo = {}, set()
            for v in sched["order"]:
                if ops[v] == "input":
                    continue
                s = sched["stream_of"][v]
                if s in last:
                    fifo.add((last[s], v))
                last[s] = v
            lam = {(a, b) for a, b in sched["sync"] if ops[a] != "input"}
            assert set(ge) == fifo | lam, (name, assignment)


def test_multi_stream_graph_edges_of_a_training_graph_with_gathered_updates():
    """Weight updates that nothing reads have no launch of their own: the last update of a stream
    carries out those before it on that stream. The graph must still order every tensor an update
    reads (gradient, and the readers of the weights it is told to run after) before the launch
    that stands in for it."""
    fwd = workloads.nas_cell_cifar(batch=2)
    out = fwd.outputs[0]
    w = workloads.training_graph(fwd, 1e-6, {out: np.zeros(fwd.nodes[out].shape, np.float32)})
    ops = [nd.op for nd in w.nodes]
    updates = [v for v in range(len(ops)) if ops[v] == "sgd_update"]
    assert len(updates) > 10
    for fuse in (True, False):
        r = GraphRunner(w)
        sched = r.schedule()
        r.plan()
        launched_by, ge = B.ng_get_graph_edges(r.g, fuse)
        r.close()
        ok, why = _graph_order_is_safe(w, launched_by, ge)
        assert ok, (fuse, why)
        if not fuse:
            assert all(launched_by[v] == v for v in updates)
            continue
        pos = {v: i for i, v in enumerate(sched["order"])}
        for s in set(sched["stream_of"][v] for v in updates):
            mine = [v for v in updates if sched["stream_of"][v] == s]
            last = max(mine, key=lambda v: pos[v])
            assert all(launched_by[v] == last for v in mine), s
        # planted mistake: without the edges into one of the standing-in launches the check fails
        last = launched_by[updates[0]]
        broken = [e for e in ge if e[1] != last]
        assert len(broken) < len(ge) and not _graph_order_is_safe(w, launched_by, broken)[0]
    # What the single-stream modes launch: one launch for all updates, and a batch-norm's input gradient and parameter
    # gradients (same dy, same x) in one launch, that of whichever of the two comes first.
    r = GraphRunner(w)
    sched = r.schedule()
    r.plan()
    launched_by, ge = B.ng_get_graph_edges(r.g, 2)
    r.close()
    assert _graph_order_is_safe(w, launched_by, ge)[0]
    pos = {v: i for i, v in enumerate(sched["order"])}
    assert len({launched_by[v] for v in updates}) == 1 and launched_by[updates[0]] == max(updates, key=lambda v: pos[v])
    halves = [v for v in range(len(ops)) if ops[v] in ("bn_act_dgrad", "bn_act_wgrad")]
    absorbed = [v for v in halves if launched_by[v] != v]
    assert 2 * len(absorbed) == len(halves)
    for v in absorbed:
        u = launched_by[v]
        assert {ops[v], ops[u]} == {"bn_act_dgrad", "bn_act_wgrad"} and w.nodes[v].preds == w.nodes[u].preds and pos[u] < pos[v]
    # ... and the input gradient and the weight gradient of a depthwise or 1 x 1 convolution (same dy) in one launch with
    # their workgroups interleaved: the later one's inputs must all come before the earlier one
    for kind in ("dwconv", "conv1x1"):
        halves = [v for v in range(len(ops)) if ops[v] in (kind + "_dgrad", kind + "_wgrad")]
        absorbed = [v for v in halves if launched_by[v] != v]
        assert len(absorbed) >= len(halves) // 2 - 1, kind            # all but the classifier's pair (other kernels)
        for v in absorbed:
            u = launched_by[v]
            assert {ops[v], ops[u]} == {kind + "_dgrad", kind + "_wgrad"} and w.nodes[v].preds[0] == w.nodes[u].preds[0]
            assert pos[u] < pos[v] and all(pos[q] < pos[u] for q in w.nodes[v].preds)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_multi_stream_graph_edges_on_the_80_node_dags(seed):
    """Seed 12 is the DAG on which the multi-stream HIP graph was seen to run task 44 before task 2
    had finished: the edge list the library hands to the runtime orders every dependency, that one
    included, under both assignments and with and without the launch fusions."""
    w = workloads.make("random200", seed=seed, n_nodes=80, n_layers=12, max_width=10, shape=(1, 16, 14, 14))
    for assignment, fuse, sched, launched_by, ge in _exact_and_default(w):
        ok, why = _graph_order_is_safe(w, launched_by, ge)
        assert ok, (seed, assignment, fuse, why)
        # and the plain statement of the oracle for the unfused graph: FIFO + Lambda covers E
        if not fuse:
            assert checks.execution_respects_edges(len(w.nodes), w.edges, sched["stream_of"], sched["order"], sched["sync"])
    if seed == 12:
        r = GraphRunner(w)
        r.schedule(); r.plan()
        launched_by, ge = B.ng_get_graph_edges(r.g, True)
        r.close()
        assert (2, 44) in w.edges
        k2, k44 = launched_by[2], launched_by[44]
        assert checks.reachable(len(w.nodes), ge)[k2][k44]


def test_graph_edges_check_catches_a_planted_mistake():
    """The checker itself: drop one needed edge from a correct list and it must say so."""
    w = workloads.make("random200", seed=12, n_nodes=80, n_layers=12, max_width=10, shape=(1, 16, 14, 14))
    r = GraphRunner(w)
    r.schedule(); r.plan()
    launched_by, ge = B.ng_get_graph_edges(r.g, False)
    r.close()
    assert _graph_order_is_safe(w, launched_by, ge)[0]
    sched_sync = [e for e in ge if e == (launched_by[2], launched_by[44])]
    assert sched_sync, "the direct edge 2 -> 44 is part of the graph"
    broken = [e for e in ge if e != sched_sync[0]]
    assert not _graph_order_is_safe(w, launched_by, broken)[0]


def test_graph_edges_errors():
    w = workloads.make("tiny_cell")
    r = GraphRunner(w)
    with pytest.raises(B.NgError) as ei:
        B.ng_get_graph_edges(r.g)
    assert ei.value.code == B.NG_ESTATE
    r.schedule(); r.plan()
    n_e = C.c_int()
    src, dst = (C.c_int * 1)(), (C.c_int * 1)()
    assert B.lib.ng_get_graph_edges(r.g, 1, None, C.byref(n_e), src, dst, 1) == B.NG_ENOMEM and n_e.value > 1
    assert B.lib.ng_get_graph_edges(r.g, 1, None, C.byref(n_e), None, None, 5) == B.NG_EINVAL
    B.ng_set_launch_fusion(r.g, False)
    r.close()


# ---- the DAG of a training iteration (forward + backward + update as tasks) -------------------

def _training_workloads():
    fw = workloads.make("tiny_cell")
    out = fw.outputs[0]
    yield workloads.training_graph(fw, 0.1, {out: np.ones(fw.nodes[out].shape, np.float32)})
    fw = workloads.nas_cell_cifar(batch=2, c=8, image=8)
    out = fw.outputs[0]
    yield workloads.training_graph(fw, 0.1, {out: np.ones(fw.nodes[out].shape, np.float32)})


def test_training_dag_registers_schedules_and_orders_every_weight_update():
    for tw in _training_workloads():
        n = len(tw.nodes)
        r = GraphRunner(tw)
        for v, nd in enumerate(tw.nodes):                        # the library's shape inference agrees with the recipe
            assert B.ng_node_shape(r.g, v) == tuple(nd.shape), (v, nd.op)
        sched = r.schedule()
        o = oracle_schedule(n, tw.edges)
        assert_same_schedule(sched, B.ng_get_scaffold(r.g), o)
        assert checks.execution_respects_edges(n, tw.edges, sched["stream_of"], sched["order"], sched["sync"])
        r.plan()
        for fuse in (True, False):
            launched_by, ge = B.ng_get_graph_edges(r.g, fuse)
            ok, why = _graph_order_is_safe(tw, launched_by, ge)
            assert ok, (tw.name, fuse, why)
            others = {tw.nodes[v].op for v in range(n) if tw.nodes[v].op != "input" and launched_by[v] != v}
            # without fusion every task has its launch; with it only weight updates (gathered per stream), the halves of a
            # batch-norm's backward pass and a batch-norm behind a 1 x 1 convolution may ride on another task's launch
            assert others <= ({"sgd_update", "bn_act", "bn_act_dgrad", "bn_act_wgrad"} if fuse else set()), (tw.name, fuse, others)
        plan = B.ng_resident_dry_plan(r.g)
        assert plan["ok"]
        r.close()
        # an update writes its weight in place: every other node that reads that weight must be its ancestor,
        # and nothing that reads the weight may come after it
        reach = checks.reachable(n, tw.edges)
        readers = {}
        for v, nd in enumerate(tw.nodes):
            keys = [(v, j) for j in range(len(nd.weights))] + [tuple(k) for k in nd.shared_weights]
            for k in keys:
                readers.setdefault(k, []).append(v)
        assert tw.update_of
        for key, upd in tw.update_of.items():
            for v in readers[key]:
                assert v == upd or reach[v][upd], (tw.name, key, v, upd)
        # one gradient node per forward node that has one, one update per trainable weight (batch-norm statistics stay fixed)
        for v, nd in enumerate(tw.forward.nodes):
            want = {"conv1x1": 1, "conv3x3": 1, "dwconv": 1, "fc": 2, "bn_act": 2}.get(nd.op, 0)
            assert sum(1 for (u, j) in tw.update_of if u == v) == want, (v, nd.op)


def test_training_operator_errors():
    g = B.ng_create()
    x = B.ng_add_input(g, (2, 4, 6, 6))
    dy = B.ng_add_input(g, (2, 4, 3, 3))
    p = B.ng_op_params()
    p.stride, p.pad, p.pool_mode = 1, 1, 0
    with pytest.raises(B.NgError) as ei:                          # a 3x3 stride-1 pool of x is 6x6, not 3x3
        B.ng_add_node(g, B.NG_OP_POOL_DGRAD, p, [dy, x], [])
    assert ei.value.code == B.NG_ESHAPE
    p.stride = 2
    ok = B.ng_add_node(g, B.NG_OP_POOL_DGRAD, p, [dy, x], [])
    assert B.ng_node_shape(g, ok) == (2, 4, 6, 6)
    q = B.ng_op_params()
    q.cout, q.lr = 1000, 0.1
    with pytest.raises(B.NgError) as ei:                          # more elements than the gradient tensor has
        B.ng_add_node(g, B.NG_OP_SGD_UPDATE, q, [ok], [0])
    assert ei.value.code == B.NG_ESHAPE
    q.cout = 10
    with pytest.raises(B.NgError):                                # an update needs exactly one weight buffer
        B.ng_add_node(g, B.NG_OP_SGD_UPDATE, q, [ok], [])
    s = B.ng_op_params()
    s.cout = 6
    s.slice_lo[0], s.slice_hi[0], s.slice_lo[1] = 1, 4, 4          # 3 channels to [4, 7) of 6: out of range
    with pytest.raises(B.NgError) as ei:
        B.ng_add_node(g, B.NG_OP_SLICE_PAD, s, [dy], [])
    assert ei.value.code == B.NG_ESHAPE
    s.slice_lo[1] = 3
    assert B.ng_node_shape(g, B.ng_add_node(g, B.NG_OP_SLICE_PAD, s, [dy], [])) == (2, 6, 3, 3)
    B.ng_destroy(g)


# ---- which hand-written kernel a node is bound to (decided on the host from shapes alone) --------------------------
def _planned_kernels(w):
    r = GraphRunner(w)
    try:
        r.schedule()
        r.plan()
        return [B.ng_planned_task_kernel(r.g, v) for v in range(len(w.nodes))]
    finally:
        r.close()


def _single_ops(build):
    b = Builder("single_op")
    build(b)
    rng = np.random.default_rng(0)
    b.draw_weights(rng, 0.2, "random")
    return b.finish(rng)


def _kernels_on(shape, ops):
    """Kernel names of `ops` (callables taking the builder and the input node) applied to one input of `shape`."""
    def build(b):
        x = b.input(*shape)
        for op in ops:
            op(b, x)
    return _planned_kernels(_single_ops(build))[1:]


def test_kernel_choice_of_the_patch_stationary_convolutions():
    def c3(cout, stride=1, pad=1):
        return lambda b, x: b.conv3x3(x, cout, stride, pad)
    # 96 rows: 640 tiles (3 rounds) against 1280 of 64 rows (5 rounds); 64 rows; 32 output channels: 32 x 128 tiles, whose runs
    # of 128 pixels need a patch of 259; stride 2: every second pixel of a patch of 385
    assert _kernels_on((32, 96, 35, 35), [c3(96), c3(64), c3(32), c3(96, 2, 0)]) == [
        "conv3x3_patch_96x64", "conv3x3_patch_64x64", "conv3x3_patch_32x128_wide", "conv3x3_patch_64x64_wide"]
    # 480 tiles of 64 rows (2 rounds) against 320 of 96 (2 rounds of 1.5 x the work)
    assert _kernels_on((32, 192, 17, 17), [c3(192)]) == ["conv3x3_patch_64x64"]
    # 256 tiles of 96 rows: one per compute unit
    assert _kernels_on((32, 384, 8, 8), [c3(768)]) == ["conv3x3_patch_96x64"]
    # wide rows and thousands of tiles: 64 x 128
    assert _kernels_on((32, 32, 147, 147), [c3(64)]) == ["conv3x3_patch_64x128_wide"]
    # 24 input channels are not whole blocks of 16; a run of 64 pixels of a 299-wide image can need 4 x 301 pixels of patch
    assert _kernels_on((2, 24, 97, 96), [c3(40)]) == ["conv3x3_lds_64x64"]
    assert _kernels_on((1, 16, 299, 299), [c3(64)]) == ["conv3x3_lds_64x64"]
    # 1225 output pixels: a small problem
    assert _kernels_on((1, 96, 35, 35), [c3(96)])[0].startswith("conv3x3_mfma_")


def test_kernel_choice_of_conv1x1_pool_and_the_networks():
    def pw(cout):
        return lambda b, x: b.conv1x1(x, cout)

    def pool(mode, stride, pad):
        return lambda b, x: b.pool(x, mode, stride, pad)
    assert _kernels_on((32, 768, 17, 17), [pw(192)]) == ["conv1x1_patch_64x64"]          # 435 tiles of 64 x 64
    assert _kernels_on((32, 1280, 8, 8), [pw(192)]) == ["conv1x1_patch_32x64"]           # 96 tiles of 64 x 64: 32-row tiles instead
    assert _kernels_on((5, 37, 45, 47), [pw(150)]) == ["conv1x1_mfma_64x64"]             # 37 input channels: the LDS-tiled kernel
    small = _kernels_on((1, 768, 17, 17), [pw(192), pool("max", 1, 1)])                  # 289 columns: small problems
    assert not small[0].startswith("conv1x1_patch") and small[1] == "pool3x3"
    assert _kernels_on((32, 288, 35, 35), [pool("max", 1, 1), pool("avg", 2, 0)]) == ["pool3x3_col4_s1", "pool3x3_col4_s2"]
    # the Inception-style network at batch 32: every convolution but the 3-channel stem on the patch kernels
    w = workloads.make("inception_style", batch=32)
    k = _planned_kernels(w)
    convs = [k[v] for v, nd in enumerate(w.nodes) if nd.op in ("conv1x1", "conv3x3")]
    assert sorted(c for c in convs if not c.startswith(("conv1x1_patch", "conv3x3_patch"))) == ["conv3x3_t16s2"]
    # at batch 1 only its wide stem layers have 2048 output pixels
    w1 = workloads.make("inception_style")
    k1 = _planned_kernels(w1)
    assert sum(c.startswith(("conv1x1_patch", "conv3x3_patch")) for c in k1) == 4
    # errors
    r = GraphRunner(w)
    try:
        with pytest.raises(B.NgError):
            B.ng_planned_task_kernel(r.g, 0)                                                    # not planned yet
        r.schedule()
        r.plan()
        with pytest.raises(B.NgError):
            B.ng_planned_task_kernel(r.g, len(w.nodes))
    finally:
        r.close()


def test_kernel_choice_in_a_training_graph():
    fwd = workloads.nas_cell_cifar(batch=32)
    out = fwd.outputs[0]
    w = workloads.training_graph(fwd, 1e-6, {out: np.zeros(fwd.nodes[out].shape, np.float32)})
    k = _planned_kernels(w)
    by_op = {}
    for v, nd in enumerate(w.nodes):
        by_op.setdefault(nd.op, set()).add(k[v])
    # weights change between replays: convolutions read the weights as they are, never a repacked copy; with 44 and 88
    # channels the 1 x 1 convolutions stream the pixels 128 bits at a time, forward and input gradient
    assert by_op["conv1x1"] == {"conv1x1_px_fwd"} and by_op["conv3x3"] == {"gemm_conv3x3_fwd"}
    # tensors of 1.4 M elements: pooling with four outputs of a column per thread (0.7 M in the reduction cell: one per thread);
    # depthwise convolutions, forward and backward, on whole 32 x 32 or 16 x 16 planes staged in LDS
    assert by_op["pool"] == {"pool3x3", "pool3x3_col4_s1"}
    assert by_op["dwconv"] == {"dwconv_lds"} and by_op["dwconv_dgrad"] == {"dwconv_dgrad_lds"} and by_op["dwconv_wgrad"] == {"dwconv_wgrad"}
    # the classifier (1 x 1 maps, 10 x 264 weights, a bias): three GEMMs of a few thousand outputs, no tiles
    assert by_op["conv1x1_dgrad"] == {"conv1x1_px_dgrad", "small_gemm"} and by_op["fc"] == {"small_gemm"}
    assert sum(name == "small_gemm" for name in k) == 3
    assert by_op["pool_dgrad"] == {"pool3x3_dgrad_lds"}
    # 32 x 32 and 16 x 16 maps: the weight gradient reads both operands 128 bits along the pixels; the fc (1 x 1 maps) cannot
    assert by_op["conv1x1_wgrad"] == {"conv1x1_wgrad_px_16", "conv1x1_wgrad_px_32", "small_gemm"}
    assert by_op["conv3x3_wgrad"] == {"conv3x3_wgrad_px_16"}         # the stem: 44 x 27 weights, rows of 32 pixels
