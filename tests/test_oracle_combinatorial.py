"""Pins for the checker's integer read-out steps (CPU only)."""
import numpy as np
import pytest

from oracle import combinatorial as cb
from tests import helpers as hp


def test_rounding_rule_at_the_threshold():
    p = np.array([0.0, 0.49999997, 0.5, 0.50000006, 1.0], dtype=np.float32)
    np.testing.assert_array_equal(cb.round_probs(p), [0, 0, 1, 1, 1])


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("scope", ["local", "all"])
def test_repair_equals_exhaustive_definition(seed, scope):
    rs = np.random.RandomState(seed)
    n, P = 12, 2
    edges = hp.random_graph(n, 0.35, rs)
    part = rs.randint(0, P, n).astype(np.int32)
    rowptr, col = hp.csr_from_edges(n, edges)
    # coarse probabilities so that ties occur and the id tie-break matters
    p = (rs.randint(0, 6, n) / 5.0).astype(np.float32)
    x = cb.round_probs(p)
    got = cb.repair(n, rowptr, col, part, p, x, scope)
    order = sorted(range(n), key=lambda i: (-float(p[i]), i))
    scoped = edges if scope == "all" else [(u, v) for u, v in edges if part[u] == part[v]]
    want = hp.lexicographically_first_independent_subset(n, scoped, order, x)
    np.testing.assert_array_equal(got, want)
    # independent in scope, subset of x, maximal within x, idempotent
    assert cb.count_conflicts(n, rowptr, col, part, got, scope) == 0
    assert (got <= x).all()
    nb = hp.adjacency_masks(n, scoped)
    kept = sum(1 << i for i in range(n) if got[i])
    for i in range(n):
        if x[i] and not got[i]:
            assert nb[i] & kept
    np.testing.assert_array_equal(cb.repair(n, rowptr, col, part, p, got, scope), got)


def test_repair_on_textbook_graphs():
    for n, edges, size in [(6, hp.complete(6), 1), (7, hp.star(7), 6), (8, hp.cycle(8), 4)]:
        rowptr, col = hp.csr_from_edges(n, edges)
        p = np.full(n, 0.9, dtype=np.float32)
        if edges == hp.star(7):
            p[0] = 0.6            # centre has the lowest priority: all leaves survive
        y = cb.repair(n, rowptr, col, None, p, cb.round_probs(p), "all")
        assert y.sum() == size <= hp.independence_number(n, edges)


@pytest.mark.parametrize("seed", range(4))
def test_cut_edges_invariants(seed):
    rs = np.random.RandomState(seed)
    n, P = 40, 4
    edges = hp.random_graph(n, 0.15, rs)
    part = rs.randint(0, P, n).astype(np.int32)
    rowptr, col = hp.csr_from_edges(n, edges)
    u, v = cb.cut_edges(n, rowptr, col, part)
    want = sorted((a, b) for a, b in edges if part[a] != part[b])
    assert list(zip(u.tolist(), v.tolist())) == want            # sorted, u < v, unique
    local = [(a, b) for a, b in edges if part[a] == part[b]]
    assert len(want) + len(local) == len(edges)
    u2, v2 = cb.cut_edges_vectorised(n, rowptr, col, part)
    np.testing.assert_array_equal(u, u2)
    np.testing.assert_array_equal(v, v2)
    c = cb.cross_mask(n, u, v)
    touched = {a for e in want for a in e}
    np.testing.assert_array_equal(c, [1 if i in touched else 0 for i in range(n)])
    # one subgraph: nothing is cut
    u0, v0 = cb.cut_edges(n, rowptr, col, np.zeros(n, dtype=np.int32))
    assert len(u0) == 0 and cb.cross_mask(n, u0, v0).sum() == 0
    # conflicts among the cut edges
    x = (rs.random(n) < 0.5).astype(np.uint8)
    cu, cv = cb.conflict_edges(u, v, x)
    assert list(zip(cu.tolist(), cv.tolist())) == [e for e in want if x[e[0]] and x[e[1]]]
    assert cb.count_conflicts(n, rowptr, col, part, x, "all") == \
        sum(1 for a, b in edges if x[a] and x[b])
    assert cb.count_conflicts(n, rowptr, col, part, x, "local") == \
        sum(1 for a, b in local if x[a] and x[b])
    assert cb.cut_value(n, rowptr, col, part, x, "all") == sum(1 for a, b in edges if x[a] != x[b])
    assert cb.cut_value(n, rowptr, col, part, x, "local") == sum(1 for a, b in local if x[a] != x[b])
