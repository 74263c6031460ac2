"""Seeded random DAGs for scheduler tests (structure only, no arithmetic)."""
import numpy as np


def random_dag(rng: np.random.Generator, n: int, p: float, max_in: int = 8):
    """Edges (u, v) with u < v; each earlier node is a predecessor with probability p,
    at most ``max_in`` predecessors per node."""
    edges = []
    for v in range(1, n):
        cand = [u for u in range(v) if rng.random() < p]
        if len(cand) > max_in:
            cand = sorted(int(c) for c in rng.choice(cand, size=max_in, replace=False))
        edges += [(u, v) for u in cand]
    return edges


def layered_dag(rng: np.random.Generator, n_layers: int, max_width: int, max_in: int = 3):
    """A layered DAG like the random benchmark config: node 0 feeds layer 0, later
    nodes pick 1..max_in predecessors from earlier layers."""
    edges, earlier, n = [], [], 1
    for li in range(n_layers):
        layer = []
        for _ in range(int(rng.integers(1, max_width + 1))):
            v = n
            n += 1
            if li == 0:
                preds = [0]
            else:
                k = min(int(rng.integers(1, max_in + 1)), len(earlier))
                preds = sorted(int(x) for x in rng.choice(earlier, size=k, replace=False))
            edges += [(u, v) for u in preds]
            layer.append(v)
        earlier += layer
    return n, edges
