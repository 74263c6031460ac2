"""Safety of a static memory plan under multi-stream execution (test infrastructure, see package doc).

The method fixes every tensor's address ahead of time (Section 4.1: the memory a run needs is
the same every time, so it is reserved once). When two tensors share bytes of that memory the
plan is safe only if no execution the schedule allows can write one of them while the other is
still needed. The schedule (Section 4.2, Appendix A) guarantees exactly the order of the DAG:
a task starts after all its predecessors; tasks that are not ordered by the DAG may run in any
order or at the same time.

Two formulations, checked against each other in the tests:

* by definition: run every linear extension of the DAG (tiny DAGs only); a step that writes
  bytes of a tensor which a not yet executed task still reads, or which is a network output or
  the input, is a violation. (Tasks that overlap in time are covered: if a and b are unordered,
  both orders occur among the extensions.)
* by reachability: tensors a and b that share bytes are safe iff a's producer and all of a's
  readers are ancestors of b's producer, or the same with a and b exchanged. Tensors that the
  plan deliberately nests (an input of a concat produced in place inside the concat's result)
  are told apart from clashes by `nested_ok`.

A result that nobody reads is a network output and belongs in `keep` (the two formulations
differ on never-read tensors that are not kept: by definition nothing needs them, while the
reachability rule still refuses to let two unordered tasks write the same bytes).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

Edge = Tuple[int, int]


def _ancestors(n: int, edges: Sequence[Edge]) -> List[int]:
    preds = [[] for _ in range(n)]
    for u, v in edges:
        preds[v].append(u)
    anc = [0] * n
    for v in range(n):                       # ids are a topological order
        for u in preds[v]:
            anc[v] |= anc[u] | (1 << u)
    return anc


def overlapping_pairs(offset: Sequence[int], nbytes: Sequence[int]) -> List[Tuple[int, int]]:
    n = len(offset)
    return [(a, b) for a in range(n) for b in range(a + 1, n)
            if nbytes[a] and nbytes[b] and offset[a] < offset[b] + nbytes[b] and offset[b] < offset[a] + nbytes[a]]


def plan_is_safe(n: int, edges: Sequence[Edge], offset, nbytes, keep: Sequence[int] = (),
                 nested_ok=lambda a, b: False) -> bool:
    """Reachability formulation. `keep`: tensors that must survive the whole run (network input
    and outputs); they may not share bytes with anything."""
    edges = sorted(set(edges))
    anc = _ancestors(n, edges)
    readers = [[] for _ in range(n)]
    for u, v in edges:
        readers[u].append(v)

    def dead_for(a: int, b: int) -> bool:     # everything that touches tensor a precedes task b
        return all((anc[b] >> x) & 1 for x in [a] + readers[a])

    for a, b in overlapping_pairs(offset, nbytes):
        if nested_ok(a, b):
            continue
        if a in keep or b in keep:
            return False
        if not (dead_for(a, b) or dead_for(b, a)):
            return False
    return True


def plan_is_safe_by_definition(n: int, edges: Sequence[Edge], offset, nbytes, keep: Sequence[int] = ()) -> bool:
    """Every linear extension of the DAG, step by step (n <= 9 or so)."""
    edges = sorted(set(edges))
    preds = [[] for _ in range(n)]
    readers = [[] for _ in range(n)]
    for u, v in edges:
        preds[v].append(u)
        readers[u].append(v)
    clash = {v: [] for v in range(n)}
    for a, b in overlapping_pairs(offset, nbytes):
        clash[a].append(b)
        clash[b].append(a)
    for a, b in overlapping_pairs(offset, nbytes):
        if a in keep or b in keep:
            return False

    def run(done: int) -> bool:
        if done == (1 << n) - 1:
            return True
        for v in range(n):
            if (done >> v) & 1 or any(not (done >> u) & 1 for u in preds[v]):
                continue
            # v writes its tensor now: nothing that shares its bytes may still be needed
            # (the opposite case, z written later while v's tensor is needed, shows up at z's step)
            for z in clash[v]:
                if (done >> z) & 1 and any(not (done >> r) & 1 for r in readers[z]):
                    return False             # z is live: a reader of z has not run yet
            if not run(done | (1 << v)):
                return False
        return True

    return run(0)
