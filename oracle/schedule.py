"""Stream assignment and synchronisation plan (test infrastructure, see package doc).

Follows Algorithm 1 of the paper (Section 4.2) in its own order and notation:
G = (V, E) with nodes 0..V-1 in topological (registration) order, G' = (V, E')
its minimum equivalent graph, B the bipartite graph of E', M a maximum
matching, chains = the sets of Steps 4-5. The synchronisation plan Lambda and
its count follow Appendix A (safe plans, Lemma 4, Theorem 3).

The paper leaves these points open; the readings taken here are:

* Which maximum matching (Step 3): augmenting-path search ("Ford-Fulkerson"
  with unit capacities), left nodes tried in ascending id, candidate right
  nodes in ascending id.
* Step 2 takes E' (Algorithm 1) while the complexity paragraph of Appendix A
  speaks of the transitive closure. Run on E' alone the chains are a minimum
  path cover of G', which can be wider than the widest antichain. Here the
  E' matching is kept (Theorems 3 and 4 hold for it) and chains are then joined
  tail-to-head through closure edges (phase 2: such a merge adds no same-stream
  E' edge and removes none, so the synchronisation count of Lemma 4 is
  unchanged), and a last augmenting pass over the whole closure (phase 3,
  normally a no-op) guarantees that the number of streams equals the maximum
  antichain width.
* Stream labels (irrelevant to the theorems): scan nodes in ascending id, a
  chain gets the next label when its first node is met.
* Submission order: ascending node id. One event per producer that has at
  least one cross-stream E' successor; a consumer waits before it is launched.
"""
from __future__ import annotations

import sys
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

Edge = Tuple[int, int]


def transitive_closure(n: int, edges: Sequence[Edge]) -> List[int]:
    """reach[u] = bitmask of nodes reachable from u by a non-empty path."""
    succ = [[] for _ in range(n)]
    for u, v in edges:
        assert 0 <= u < v < n, "edges must go from a smaller to a larger id"
        succ[u].append(v)
    reach = [0] * n
    for u in range(n - 1, -1, -1):
        for v in succ[u]:
            reach[u] |= (1 << v) | reach[v]
    return reach


def minimum_equivalent_graph(n: int, edges: Sequence[Edge], reach: List[int]) -> List[Edge]:
    """Step 1. For a DAG the MEG is unique: keep (u, v) iff no node w lies
    strictly between them (u reaches w and w reaches v)."""
    anc = [0] * n                       # anc[v] = nodes that reach v
    for u in range(n):
        r, v = reach[u], 0
        while r:
            if r & 1:
                anc[v] |= 1 << u
            r >>= 1
            v += 1
    return sorted({(u, v) for u, v in edges if reach[u] & anc[v] == 0})


def _augment(lefts, adj, match_l: Dict[int, int], match_r: Dict[int, int]) -> None:
    """Augmenting-path maximum matching; extends match_l/match_r in place."""
    def attempt(x, seen) -> bool:
        for y in adj[x]:
            if y in seen:
                continue
            seen.add(y)
            if y not in match_r or attempt(match_r[y], seen):
                match_l[x] = y
                match_r[y] = x
                return True
        return False

    old = sys.getrecursionlimit()
    sys.setrecursionlimit(max(old, 4 * len(adj) + 1000))
    try:
        for x in lefts:
            if x not in match_l:
                attempt(x, set())
    finally:
        sys.setrecursionlimit(old)


def _label_chains(n: int, nxt: Dict[int, int]) -> List[int]:
    """Label the paths of a matching (x -> nxt[x]) in order of their first node."""
    label = [-1] * n
    count = 0
    for v in range(n):
        if label[v] < 0:                # v is the first node of an unlabelled path
            w = v
            while True:
                label[w] = count
                if w not in nxt:
                    break
                w = nxt[w]
            count += 1
    return label


def _bits(mask: int) -> List[int]:
    out, i = [], 0
    while mask:
        if mask & 1:
            out.append(i)
        mask >>= 1
        i += 1
    return out


@dataclass
class Schedule:
    n: int
    reach: List[int]
    meg: List[Edge]                 # E', sorted
    matching: List[Edge]            # M of Step 3 on E', sorted
    chain_of: List[int]             # Steps 4-5 verbatim
    n_chains: int
    stream_of: List[int]            # after joining chains down to the antichain width
    n_streams: int
    sync: List[Edge]                # Lambda, sorted: cross-stream E' edges
    event_of: List[int]             # event id of a producer in Lambda, else -1
    n_events: int
    order: List[int]                # submission order
    waits: List[List[int]]          # waits[v] = producers v waits for, ascending
    fork: List[int]                 # non-origin streams whose first task has no wait
    join: List[int]                 # non-origin streams the origin waits for at the end
    phase3_changed: bool


def schedule(n: int, edges: Sequence[Edge]) -> Schedule:
    edges = sorted(set(edges))
    reach = transitive_closure(n, edges)
    meg = minimum_equivalent_graph(n, edges, reach)

    # Steps 2-3: maximum matching of B = (V1, V2, {(x_i, y_j) : (v_i, v_j) in E'}).
    adj1 = [[] for _ in range(n)]
    for u, v in meg:
        adj1[u].append(v)
    match_l: Dict[int, int] = {}
    match_r: Dict[int, int] = {}
    _augment(range(n), adj1, match_l, match_r)
    matching = sorted(match_l.items())

    # Steps 4-5: merge the sets of v_i and v_j for each matched pair (union-find).
    parent = list(range(n))

    def find(a):
        while parent[a] != a:
            a = parent[a]
        return a
    for u, v in matching:
        parent[find(v)] = find(u)
    chain_of, seen = [-1] * n, {}
    for v in range(n):
        chain_of[v] = seen.setdefault(find(v), len(seen))
    n_chains = len(seen)

    # Phase 2: join chain tails to chain heads they reach; the E' matching is not touched.
    tails = [v for v in range(n) if v not in match_l]
    heads = {v for v in range(n) if v not in match_r}
    adj2 = {t: [h for h in _bits(reach[t]) if h in heads] for t in tails}
    _augment(tails, adj2, match_l, match_r)

    # Phase 3: augment over the full closure so that #paths = maximum antichain
    # (Dilworth / Fulkerson). E' successors are tried first.
    before = dict(match_l)
    adj3 = [adj1[u] + [v for v in _bits(reach[u]) if v not in adj1[u]] for u in range(n)]
    _augment(range(n), adj3, match_l, match_r)
    phase3_changed = match_l != before

    stream_of = _label_chains(n, match_l)
    n_streams = max(stream_of) + 1 if n else 0

    # Appendix A: every E' edge is the only path between its ends (Lemma 1), so a
    # cross-stream E' edge must be synchronised itself; same-stream ones need nothing.
    sync = [(u, v) for u, v in meg if stream_of[u] != stream_of[v]]
    event_of = [-1] * n
    for i, u in enumerate(sorted({u for u, _ in sync})):
        event_of[u] = i
    n_events = sum(e >= 0 for e in event_of)
    waits = [[] for _ in range(n)]
    for u, v in sync:
        waits[v].append(u)

    # Capture scaffolding (not part of Lambda): stream 0 is the origin.
    first = {}
    for v in range(n):
        first.setdefault(stream_of[v], v)
    fork = sorted(s for s, v in first.items() if s != 0 and not waits[v])
    join = sorted(s for s in first if s != 0)

    return Schedule(n, reach, meg, matching, chain_of, n_chains, stream_of, n_streams, sync,
                    event_of, n_events, list(range(n)), waits, fork, join, phase3_changed)


# ---------------------------------------------------------------------------------------
# The jointly optimal assignment: fewest streams, and among those fewest synchronisations
# ---------------------------------------------------------------------------------------
# Definition (Section 4.2 states the two goals; Appendix A counts synchronisations): a stream
# assignment with maximum logical concurrency puts two nodes on one stream only if one reaches
# the other, so every stream is a chain of the closure; the number of streams is at least the
# widest antichain; a safe plan must synchronise exactly the E' edges whose ends sit on
# different streams (Lemma 1, Lemma 4). "Exact" = a partition of V into chains that has the
# fewest chains and, among all such partitions, the fewest cross-chain E' edges.

def _is_chain(nodes: Sequence[int], reach: List[int]) -> bool:
    nodes = sorted(nodes)
    return all((reach[a] >> b) & 1 for a, b in zip(nodes, nodes[1:]))


def exact_optimum_by_enumeration(n: int, edges: Sequence[Edge]) -> Tuple[int, int]:
    """(fewest streams, fewest synchronisations at that stream count) by trying every partition
    of the nodes into sets (tiny n only: Bell(9) = 21147 partitions)."""
    edges = sorted(set(edges))
    reach = transitive_closure(n, edges)
    meg = minimum_equivalent_graph(n, edges, reach)
    best = None

    def place(v: int, blocks: List[List[int]]):
        nonlocal best
        if v == n:
            label = {}
            for i, b in enumerate(blocks):
                for x in b:
                    label[x] = i
            key = (len(blocks), sum(label[a] != label[b] for a, b in meg))
            if best is None or key < best:
                best = key
            return
        for b in blocks:                         # nodes arrive in ascending id: v joins a chain iff its last node reaches v
            if (reach[b[-1]] >> v) & 1:
                b.append(v)
                place(v + 1, blocks)
                b.pop()
        blocks.append([v])
        place(v + 1, blocks)
        blocks.pop()

    place(0, [])
    return best


def schedule_exact(n: int, edges: Sequence[Edge]) -> Schedule:
    """Same record as `schedule`, with the streams of the jointly optimal assignment.

    A partition into chains is a set of vertex-disjoint paths in the closure, i.e. a matching of
    the bipartite graph whose pairs are the closure's (u, v); it has V - |matching| chains, and a
    same-stream E' edge is always a matched pair (nothing lies between its ends). So the optimum
    is a maximum matching with as many E' pairs as possible: an assignment problem in which a
    closure pair is worth V + 1, an E' pair one more, anything else nothing (solved by the
    library routine scipy.optimize.linear_sum_assignment)."""
    import numpy as np
    from scipy.optimize import linear_sum_assignment

    base = schedule(n, edges)
    reach, meg = base.reach, base.meg
    worth = np.zeros((n, n), dtype=np.int64)
    for u in range(n):
        for v in _bits(reach[u]):
            worth[u, v] = n + 1
    for u, v in meg:
        worth[u, v] += 1
    rows, cols = linear_sum_assignment(worth, maximize=True)
    nxt = {int(u): int(v) for u, v in zip(rows, cols) if worth[u, v] > 0}
    stream_of = _label_chains(n, nxt)
    n_streams = max(stream_of) + 1 if n else 0
    sync = [(u, v) for u, v in meg if stream_of[u] != stream_of[v]]
    event_of = [-1] * n
    for i, u in enumerate(sorted({u for u, _ in sync})):
        event_of[u] = i
    waits = [[] for _ in range(n)]
    for u, v in sync:
        waits[v].append(u)
    first = {}
    for v in range(n):
        first.setdefault(stream_of[v], v)
    fork = sorted(s for s, v in first.items() if s != 0 and not waits[v])
    join = sorted(s for s in first if s != 0)
    return Schedule(n, reach, meg, base.matching, base.chain_of, base.n_chains, stream_of, n_streams, sync,
                    event_of, sum(e >= 0 for e in event_of), list(range(n)), waits, fork, join, False)
