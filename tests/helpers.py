"""Small graphs and brute-force routines used by the checker's pins.

Nothing here imports the checker or the device library."""
import itertools

import numpy as np


def csr_from_edges(n, edges):
    adj = [set() for _ in range(n)]
    for u, v in edges:
        if u != v:
            adj[u].add(v)
            adj[v].add(u)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    col = []
    for i in range(n):
        col.extend(sorted(adj[i]))
        rowptr[i + 1] = len(col)
    return rowptr, np.asarray(col, dtype=np.int32)


def random_graph(n, p, rs):
    return [(i, j) for i in range(n) for j in range(i + 1, n) if rs.random() < p]


def path(n):
    return [(i, i + 1) for i in range(n - 1)]


def cycle(n):
    return path(n) + [(n - 1, 0)]


def complete(n):
    return list(itertools.combinations(range(n), 2))


def star(n):
    return [(0, i) for i in range(1, n)]


def adjacency_masks(n, edges):
    nb = [0] * n
    for u, v in edges:
        nb[u] |= 1 << v
        nb[v] |= 1 << u
    return nb


def independence_number(n, edges):
    nb = adjacency_masks(n, edges)
    best = 0
    for s in range(1 << n):
        ok = True
        t = s
        while t:
            i = (t & -t).bit_length() - 1
            if nb[i] & s:
                ok = False
                break
            t &= t - 1
        if ok:
            best = max(best, bin(s).count("1"))
    return best


def max_cut(n, edges):
    best = 0
    for s in range(1 << (n - 1)):
        c = sum(1 for u, v in edges if ((s >> u) & 1) != ((s >> v) & 1))
        best = max(best, c)
    return best


def lexicographically_first_independent_subset(n, edges, order, selected):
    """By exhaustion: among ALL independent subsets of the selected nodes, the one
    whose indicator sequence read along `order` is lexicographically largest
    (i.e. it keeps the earliest possible nodes).  No greedy walk is used."""
    nb = adjacency_masks(n, edges)
    sel = [i for i in order if selected[i]]
    best_key, best_set = None, 0
    for bits in range(1 << len(sel)):
        s = 0
        for b, i in enumerate(sel):
            if (bits >> b) & 1:
                s |= 1 << i
        if any((nb[i] & s) for i in sel if (s >> i) & 1):
            continue
        key = tuple((s >> i) & 1 for i in sel)
        if best_key is None or key > best_key:
            best_key, best_set = key, s
    return np.array([(best_set >> i) & 1 for i in range(n)], dtype=np.uint8)
