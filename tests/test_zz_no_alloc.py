"""The replay entry point that allocates nothing (ng_replay_static) against ng_replay in the
device-resident mode: same recorded plan, same kernel, completion counters in the library's static
device array instead of memory from hipMalloc - every tensor must come out bit for bit the same.
Two calls in a row share the array, the second on a smaller graph; then the first graph again."""
import numpy as np
import pytest

import workloads
from workloads.model import Builder
from paper_2012_02732_amd import GraphRunner, binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _every_tensor(r, w):
    return [r.output(v) for v in range(len(w.nodes))]


def _reference(r, w):
    r.arena.zero_()
    r.set_input(w.input)
    r.replay(B.NG_MODE_DEVICE_RESIDENT)
    r.sync()
    return _every_tensor(r, w)


def _static(r, w, times=1):
    r.arena.zero_()
    r.set_input(w.input)
    for _ in range(times):
        B.ng_replay_static(r.g)
        B.ng_sync(r.g)
    return _every_tensor(r, w)


def test_replay_static_equals_the_device_resident_replay_on_two_graphs_in_a_row():
    big, small = workloads.make("nasnet_style"), workloads.make("tiny_cell")
    rb, rs = GraphRunner(big, DEV), GraphRunner(small, DEV)
    rb.prepare(plan_trials=1)
    rs.prepare(plan_trials=1)
    try:
        ref_big, ref_small = _reference(rb, big), _reference(rs, small)
        got_big = _static(rb, big)                       # first call on this GPU: looks the array's address up
        got_small = _static(rs, small)                   # second call, smaller graph, same array
        for v in range(1, len(big.nodes)):
            assert np.array_equal(got_big[v], ref_big[v]), ("nasnet_style", v, big.nodes[v].op)
        for v in range(1, len(small.nodes)):
            assert np.array_equal(got_small[v], ref_small[v]), ("tiny_cell", v, small.nodes[v].op)
        again = _static(rb, big, times=3)                # the array now holds the small graph's counts: cleared by the call
        for v in range(1, len(big.nodes)):
            assert np.array_equal(again[v], ref_big[v]), ("nasnet_style again", v)
        # the ordinary replay is untouched by it (its own counters, its own replay number)
        after = _reference(rb, big)
        for v in range(1, len(big.nodes)):
            assert np.array_equal(after[v], ref_big[v])
    finally:
        rb.close()
        rs.close()


def test_replay_static_limits():
    def chain(b):
        x = b.input(1, 4, 4, 4)
        y = x
        for _ in range(1030):
            y = b.relu(y)
    b = Builder("long_chain")
    chain(b)
    rng = np.random.default_rng(0)
    b.draw_weights(rng, 0.1, "identity")
    w = b.finish(rng)
    r = GraphRunner(w, DEV)
    r.prepare(plan_trials=1, resident_xcds=1)
    try:
        with pytest.raises(B.NgError) as ei:
            B.ng_replay_static(r.g)
        assert ei.value.code == B.NG_ENOMEM and "1024" in str(ei.value)
    finally:
        r.close()
    r3 = GraphRunner(workloads.make("tiny_cell"))          # nothing captured
    with pytest.raises(B.NgError) as ei:
        B.ng_replay_static(r3.g)
    assert ei.value.code == B.NG_ESTATE
    r3.close()
