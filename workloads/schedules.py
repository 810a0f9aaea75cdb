"""Extra inputs for schedules that the method's own generator does not draw.

``random_extra_pairs``: for a general averaging matrix W_k (several disjoint pairs of
neighbours averaged in one event), a seeded random matching around each event's own pair.
These are integers handed to both sides as inputs.
"""
from __future__ import annotations

import numpy as np


def random_extra_pairs(graph, worker, neighbour, max_extra=3, seed=0):
    """For each event k: up to ``max_extra`` further edges of the graph, disjoint from each other
    and from (worker[k], neighbour[k]).  Returns (ptr[K+1] int64, a[] int32, b[] int32)."""
    rowptr, col = graph
    n = len(rowptr) - 1
    edges = [(i, int(j)) for i in range(n) for j in col[rowptr[i]:rowptr[i + 1]] if i < j]
    rng = np.random.default_rng([seed, 21])
    ptr = [0]
    a, b = [], []
    for k in range(len(worker)):
        used = {int(worker[k]), int(neighbour[k])}
        want = int(rng.integers(0, max_extra + 1))
        for e in rng.permutation(len(edges)):
            if want == 0:
                break
            u, v = edges[e]
            if u in used or v in used:
                continue
            used.update((u, v))
            if rng.integers(0, 2):
                u, v = v, u
            a.append(u)
            b.append(v)
            want -= 1
        ptr.append(len(a))
    return np.asarray(ptr, np.int64), np.asarray(a, np.int32), np.asarray(b, np.int32)


def with_identity_events(worker, neighbour, fraction=0.25, seed=0):
    """A copy of ``neighbour`` in which a random ``fraction`` of the events has neighbour = worker
    (W_k = I: the gradient is applied without averaging, as for a gradient taken from a queue)."""
    rng = np.random.default_rng([seed, 22])
    out = np.array(neighbour, np.int32)
    pick = rng.random(len(out)) < fraction
    out[pick] = np.asarray(worker, np.int32)[pick]
    return out
