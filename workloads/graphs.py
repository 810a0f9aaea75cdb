"""Communication graphs (V, E) handed to the method as CSR adjacency lists.

The paper only requires an undirected connected graph (Sec. 3.1); its own
realisations are a ring and a ring with extra 2^i + 1 hop links (Sec. 3.3.2).
"""
from __future__ import annotations

import numpy as np


def _to_csr(n, adj):
    rowptr = np.zeros(n + 1, dtype=np.int32)
    cols = []
    for i in range(n):
        rowptr[i + 1] = rowptr[i] + len(adj[i])
        cols.extend(adj[i])
    return rowptr, np.asarray(cols, dtype=np.int32)


def ring_graph(n: int):
    """Ring i <-> i +- 1 (mod n); neighbour order [i-1, i+1].  n = 2 has a single
    edge, n = 1 has none."""
    adj = []
    for i in range(n):
        nb = []
        for j in ((i - 1) % n, (i + 1) % n):
            if j != i and j not in nb:
                nb.append(j)
        adj.append(nb)
    return _to_csr(n, adj)


def hop_ring_graph(n: int):
    """Ring with the paper's extra links: i is joined to the worker 2^t + 1 hops
    away for t = 0 .. floor(log2(n-1)) (Sec. 3.3.2; base-2 logarithm and floor are
    this build's reading).  Edges are undirected; duplicates and self loops are
    dropped; neighbour lists are sorted."""
    sets = [set() for _ in range(n)]
    t = 0
    while n > 1 and (1 << t) <= n - 1:
        hop = ((1 << t) + 1) % n
        for i in range(n):
            j = (i + hop) % n
            if j != i:
                sets[i].add(j)
                sets[j].add(i)
        t += 1
    if n > 2:  # keep the plain ring links as well
        for i in range(n):
            sets[i].add((i + 1) % n)
            sets[(i + 1) % n].add(i)
    elif n == 2:
        sets[0].add(1)
        sets[1].add(0)
    return _to_csr(n, [sorted(s) for s in sets])


def random_regular4_graph(n: int, seed: int = 0):
    """Random 4-regular simple graph: the union of two seeded random Hamiltonian
    cycles, redrawn until no edge repeats (always connected)."""
    if n < 5:
        raise ValueError("need n >= 5 for a simple 4-regular graph")
    rng = np.random.default_rng(seed)
    while True:
        sets = [set() for _ in range(n)]
        ok = True
        for _ in range(2):
            perm = rng.permutation(n)
            for a, b in zip(perm, np.roll(perm, -1)):
                a, b = int(a), int(b)
                if b in sets[a]:
                    ok = False
                sets[a].add(b)
                sets[b].add(a)
        if ok and all(len(s) == 4 for s in sets):
            return _to_csr(n, [sorted(s) for s in sets])


def graph_is_valid(rowptr, col) -> bool:
    """Symmetric, no self loops, no duplicate edges, connected."""
    n = len(rowptr) - 1
    nbrs = [list(col[rowptr[i]:rowptr[i + 1]]) for i in range(n)]
    for i in range(n):
        if i in nbrs[i] or len(set(nbrs[i])) != len(nbrs[i]):
            return False
        for j in nbrs[i]:
            if j < 0 or j >= n or i not in nbrs[j]:
                return False
    seen = {0}
    stack = [0]
    while stack:
        u = stack.pop()
        for v in nbrs[u]:
            if v not in seen:
                seen.add(v)
                stack.append(v)
    return len(seen) == n
