"""Pins for the oracle's memory-plan safety check (CPU only)."""
import numpy as np

from oracle.memory import plan_is_safe, plan_is_safe_by_definition, overlapping_pairs
from dag_util import random_dag


def test_hand_cases():
    chain = (4, [(0, 1), (1, 2), (2, 3)])
    assert plan_is_safe(*chain, [0, 4, 0, 4], [4] * 4)                # tensor 0 is dead once 1 has run, 1 once 2 has run
    assert not plan_is_safe(*chain, [0, 0, 4, 8], [4] * 4)            # 1 would overwrite what it reads
    assert not plan_is_safe(*chain, [0, 4, 0, 4], [4] * 4, keep=[0])  # the network input must survive
    diamond = (4, [(0, 1), (0, 2), (1, 3), (2, 3)])
    assert not plan_is_safe(*diamond, [0, 4, 4, 8], [4] * 4)          # 1 and 2 are not ordered
    assert not plan_is_safe(*diamond, [0, 4, 8, 4], [4] * 4)          # 3 reads 1
    assert plan_is_safe(*diamond, [0, 4, 8, 0], [4] * 4)              # 0 is read by 1 and 2, both before 3
    # partial overlap counts, touching ranges do not
    assert overlapping_pairs([0, 2, 4], [4, 4, 4]) == [(0, 1), (1, 2)]
    # a reader on another branch keeps the tensor alive: 0 -> 1 -> 2, 0 -> 3 (3 unordered with 1, 2)
    fork = (4, [(0, 1), (1, 2), (0, 3)])
    assert not plan_is_safe(*fork, [0, 4, 0, 8], [4] * 4)             # 2 may run before 3 has read 0
    assert plan_is_safe(*fork, [0, 4, 4, 8], [4] * 4) is False        # 2 reads 1
    assert plan_is_safe(5, [(0, 1), (1, 2), (0, 3), (2, 4), (3, 4)], [0, 4, 8, 12, 0], [4] * 5)
    # a result nobody reads is an output: it is in `keep` and shares nothing
    assert not plan_is_safe(3, [(0, 2)], [0, 4, 4], [4, 8, 4], keep=[1, 2])


def test_reachability_formulation_equals_running_every_linear_extension():
    rng = np.random.default_rng(7)
    verdicts = {True: 0, False: 0}
    for _ in range(2500):
        n = int(rng.integers(2, 8))
        e = random_dag(rng, n, float(rng.uniform(0.2, 0.7)))
        slots = int(rng.integers(max(2, n - 3), n + 1))
        size = [int(rng.choice([4, 8])) for _ in range(n)]
        off = [int(rng.integers(0, slots)) * 4 for _ in range(n)]
        has_reader = {u for u, _ in e}
        keep = [v for v in range(n) if v not in has_reader]       # results nobody reads are the network's outputs
        if rng.random() < 0.3:
            keep.append(0)
        a = plan_is_safe(n, e, off, size, keep)
        b = plan_is_safe_by_definition(n, e, off, size, keep)
        assert a == b, (n, e, off, size, keep, a, b)
        verdicts[a] += 1
    assert verdicts[True] > 100 and verdicts[False] > 100, verdicts
