"""Checker for the integer read-out steps: rounding, conflict repair, cut edges.

TEST INFRASTRUCTURE ONLY (see oracle/gcn.py).  Plain sequential code in
ORIGINAL node order; results are exact, so the device library must agree bit
for bit.

  rounding      x_i = 1 if p_i >= 0.5 else 0                      (Sec. 3.3, binarisation rule)
  cross edge    edge (i, j) whose ends lie in different subgraphs (Sec. 3.3, first paragraph)
  cross node    a node touching a cross edge                      (Alg. 1, stage 2, mask c)
  conflict      an edge with both ends selected                   (Sec. 3.3; evaluated on x)
  error rate    conflicts / set size                              (Sec. 4.1.2)

Repair is not defined in the paper (it reports conflicts as an error rate); the
workloads ask for "threshold then greedy conflict repair".  Reading used: visit
the selected nodes in the order (p descending, id ascending) and keep a node
iff none of its neighbours (in the chosen edge scope) has been kept before it.
The result is the lexicographically first maximal independent subset of the
selected set under that order, hence unique.
"""
from __future__ import annotations

import numpy as np


def round_probs(p32: np.ndarray, thr: float = 0.5) -> np.ndarray:
    """x_i = [p_i >= thr] on float32 probabilities (the comparison is in fp32)."""
    p32 = np.asarray(p32, dtype=np.float32)
    return (p32 >= np.float32(thr)).astype(np.uint8)


def _scope_adj(n, rowptr, col, part, scope):
    """Adjacency lists restricted to the edge scope: 'local' or 'all'."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    if scope == "all" or part is None:
        return rowptr, col
    if scope != "local":
        raise ValueError(scope)
    part = np.asarray(part)
    row = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    keep = part[row] == part[col]
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row[keep], minlength=n), out=rp[1:])
    return rp, col[keep]


def count_conflicts(n, rowptr, col, part, x, scope="all") -> int:
    """Number of undirected edges in scope with both ends selected."""
    rp, cl = _scope_adj(n, rowptr, col, part, scope)
    row = np.repeat(np.arange(n, dtype=np.int64), np.diff(rp))
    both = (x[row] != 0) & (x[cl] != 0) & (row < cl)
    return int(both.sum())


def repair(n, rowptr, col, part, p32, x, scope="local") -> np.ndarray:
    """Sequential greedy repair; returns the repaired 0/1 vector (uint8)."""
    rp, cl = _scope_adj(n, rowptr, col, part, scope)
    p32 = np.asarray(p32, dtype=np.float32)
    sel = np.flatnonzero(np.asarray(x) != 0)
    # p descending, then id ascending: stable sort of ids (already ascending) by -p
    order = sel[np.argsort(-p32[sel].astype(np.float64), kind="stable")]
    kept = np.zeros(n, dtype=np.uint8)
    for i in order.tolist():
        nb = cl[rp[i]:rp[i + 1]]
        if not kept[nb].any():
            kept[i] = 1
    return kept


def cut_edges(n, rowptr, col, part):
    """(u, v) arrays of the cross edges with u < v, sorted by (u, v)."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    if part is None:
        return np.empty(0, np.int32), np.empty(0, np.int32)
    part = np.asarray(part)
    us, vs = [], []
    for i in range(n):
        for j in col[rowptr[i]:rowptr[i + 1]].tolist():
            if i < j and part[i] != part[j]:
                us.append(i)
                vs.append(j)
    return np.asarray(us, dtype=np.int32), np.asarray(vs, dtype=np.int32)


def cut_edges_vectorised(n, rowptr, col, part):
    """Same list as cut_edges, by array operations (for graphs with millions of
    edges, where the double loop above is too slow).  Pinned to cut_edges in the
    tests."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    part = np.asarray(part)
    row = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    keep = (row < col) & (part[row] != part[col])
    return row[keep].astype(np.int32), col[keep].astype(np.int32)


def cross_mask(n, u, v) -> np.ndarray:
    c = np.zeros(n, dtype=np.uint8)
    c[np.asarray(u, dtype=np.int64)] = 1
    c[np.asarray(v, dtype=np.int64)] = 1
    return c


def conflict_edges(u, v, x):
    """Subset of the listed edges with both ends selected, order kept."""
    u = np.asarray(u)
    v = np.asarray(v)
    keep = (x[u.astype(np.int64)] != 0) & (x[v.astype(np.int64)] != 0)
    return u[keep], v[keep]


def cut_value(n, rowptr, col, part, x, scope="all") -> int:
    """Max-Cut objective: edges in scope whose ends take different values."""
    rp, cl = _scope_adj(n, rowptr, col, part, scope)
    row = np.repeat(np.arange(n, dtype=np.int64), np.diff(rp))
    return int(((x[row] != x[cl]) & (row < cl)).sum())
