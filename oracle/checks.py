"""Brute-force and definitional checkers for schedules (test infrastructure).

Each function states the passage of the paper it encodes. None of them uses
the scheduling code: they take a DAG and a candidate answer and decide,
from the definitions alone, whether the answer is acceptable.
"""
from __future__ import annotations

from itertools import combinations
from typing import Iterable, List, Sequence, Tuple

Edge = Tuple[int, int]


def reachable(n: int, edges: Iterable[Edge]) -> List[List[bool]]:
    """Path relation by repeated relaxation (Floyd-Warshall style), no bit tricks."""
    r = [[False] * n for _ in range(n)]
    for u, v in edges:
        r[u][v] = True
    for k in range(n):
        for i in range(n):
            if r[i][k]:
                for j in range(n):
                    if r[k][j]:
                        r[i][j] = True
    return r


def has_max_logical_concurrency(n, edges, stream_of) -> bool:
    """Section 4.2, first goal: two nodes with no path between them never share a stream."""
    r = reachable(n, edges)
    return all(stream_of[a] != stream_of[b] or r[a][b] or r[b][a]
               for a in range(n) for b in range(a + 1, n))


def plan_is_safe(n, edges, stream_of, sync) -> bool:
    """Appendix A, definition of a safe plan: every edge (u, v) of E has both ends on
    one stream or some u->v path that contains a synchronised edge."""
    sync = set(sync)
    succ = [[] for _ in range(n)]
    for u, v in edges:
        succ[u].append(v)

    def path_with_sync(u, target, crossed):
        if u == target:
            return crossed
        return any(path_with_sync(w, target, crossed or (u, w) in sync) for w in succ[u])

    return all(stream_of[u] == stream_of[v] or path_with_sync(u, v, False) for u, v in edges)


def execution_respects_edges(n, edges, stream_of, order, sync) -> bool:
    """What the hardware guarantees (Section 2, "GPU Streams"; Section 4.2, "Stream
    Synchronization"): FIFO within a stream in submission order, plus record->wait
    pairs. Every dependency edge must follow from those orderings alone."""
    hb = []
    last = {}
    for v in order:
        s = stream_of[v]
        if s in last:
            hb.append((last[s], v))
        last[s] = v
    r = reachable(n, hb + list(sync))
    pos = {v: i for i, v in enumerate(order)}
    waits_after_records = all(pos[u] < pos[v] for u, v in sync)   # an event is recorded before it is awaited
    return waits_after_records and all(r[u][v] for u, v in edges)


def max_antichain(n, edges) -> int:
    """Largest set of pairwise unordered nodes, by enumeration (n <= ~16)."""
    r = reachable(n, edges)
    comparable = [[r[a][b] or r[b][a] for b in range(n)] for a in range(n)]
    best = 0

    def grow(start, chosen):
        nonlocal best
        best = max(best, len(chosen))
        for v in range(start, n):
            if all(not comparable[v][c] for c in chosen):
                grow(v + 1, chosen + [v])
    grow(0, [])
    return best


def min_sync_by_definition(n, edges, stream_of) -> int:
    """min_sync(G, f) of Appendix A: size of the smallest safe plan, by trying every
    subset of E in order of size (tiny graphs only)."""
    edges = sorted(set(edges))
    for k in range(len(edges) + 1):
        for plan in combinations(edges, k):
            if plan_is_safe(n, edges, stream_of, plan):
                return k
    raise AssertionError("the full edge set is always safe")


def set_partitions(items: Sequence[int]):
    """All partitions of ``items`` into non-empty blocks."""
    if not items:
        yield []
        return
    head, rest = items[0], items[1:]
    for part in set_partitions(rest):
        for i in range(len(part)):
            yield part[:i] + [[head] + part[i]] + part[i + 1:]
        yield [[head]] + part


def best_partition_sync(n, edges, sync_count) -> int:
    """Theorem 4's quantity: the least sync count over *all* stream assignments with
    maximum logical concurrency (every partition of V whose blocks are chains).
    ``sync_count(stream_of)`` supplies the count for one assignment."""
    r = reachable(n, edges)
    best = None
    for part in set_partitions(list(range(n))):
        if any(not (r[a][b] or r[b][a]) for blk in part for a, b in combinations(blk, 2)):
            continue
        f = [0] * n
        for s, blk in enumerate(part):
            for v in blk:
                f[v] = s
        c = sync_count(f)
        best = c if best is None else min(best, c)
    return best


def meg_by_edge_removal(n, edges) -> List[Edge]:
    """Minimum equivalent graph the slow way: drop an edge whenever its head stays
    reachable from its tail without it. (For a DAG the result is unique - Section
    4.2 - so any removal order gives the same set.)"""
    kept = sorted(set(edges))
    for e in list(kept):
        rest = [x for x in kept if x != e]
        if reachable(n, rest)[e[0]][e[1]]:
            kept = rest
    return kept


def lemma4_count(n, meg, stream_of) -> int:
    """|E'| - |Q(f)| with Q(f) = nodes having an E'-parent on their own stream (Lemma 4)."""
    q = {v for u, v in meg if stream_of[u] == stream_of[v]}
    return len(meg) - len(q)
