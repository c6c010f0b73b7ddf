"""Pins of the partitioning checker (oracle/louvain.py): Sec. 3.1."""
import itertools

import numpy as np
import pytest

from oracle import louvain as lv
from tests import helpers as hp


def csr(n, edges):
    return hp.csr_from_edges(n, edges)


def two_triangles():
    edges = [(0, 1), (1, 2), (0, 2), (3, 4), (4, 5), (3, 5), (2, 3)]
    return 6, edges


def test_modularity_closed_forms():
    """Two triangles joined by one edge (m = 7): each triangle has 3 inside edges and degree
    sum 7, so Q = 2 (3/7 - (7/14)^2) = 5/14.  One community for everything: Q = 0.  All
    singletons: Q = -sum (k_i / 2m)^2."""
    n, edges = two_triangles()
    rowptr, col = csr(n, edges)
    assert lv.modularity(n, rowptr, col, [0, 0, 0, 1, 1, 1]) == pytest.approx(5.0 / 14.0, abs=1e-15)
    assert lv.modularity(n, rowptr, col, [0] * 6) == pytest.approx(0.0, abs=1e-15)
    k = np.diff(rowptr)
    assert lv.modularity(n, rowptr, col, list(range(6))) == pytest.approx(-np.sum((k / 14.0) ** 2), abs=1e-15)


def test_gain_formula_is_the_modularity_difference():
    """Eq. 2 against modularity evaluated before and after the move, by definition: the node
    starts alone, then joins community c.  (Eq. 1 as printed, expanded, has k_ic / 2m in
    place of k_ic / m: it counts the community's inside weight once per direction; the
    difference of the definition decides for Eq. 2.)"""
    rs = np.random.RandomState(5)
    n = 30
    edges = hp.random_graph(n, 0.2, rs)
    rowptr, col = csr(n, edges)
    m = len(edges)
    k = np.diff(rowptr)
    base = rs.randint(0, 4, n)
    checked = 0
    for i in range(n):
        alone = base.copy()
        alone[i] = 99                                    # i in a community of its own
        q0 = lv.modularity(n, rowptr, col, alone)
        for c in range(4):
            members = [j for j in range(n) if j != i and base[j] == c]
            k_ic = sum(1 for e in range(rowptr[i], rowptr[i + 1]) if col[e] in members)
            tot_c = int(sum(k[j] for j in members))
            joined = alone.copy()
            joined[i] = c
            dq = lv.modularity(n, rowptr, col, joined) - q0
            g = lv.gain_times_2m2(m, k_ic, tot_c, int(k[i]))
            assert dq == pytest.approx(g / (2.0 * m * m), abs=1e-13)
            assert dq == pytest.approx(k_ic / m - tot_c * k[i] / (2.0 * m * m), abs=1e-13)
            checked += 1
    assert checked == 4 * n


def ring_of_cliques(q, s):
    edges = []
    for c in range(q):
        for a, b in itertools.combinations(range(s), 2):
            edges.append((c * s + a, c * s + b))
        edges.append((c * s + s - 1, ((c + 1) % q) * s))
    return q * s, edges


def test_louvain_finds_the_cliques_of_a_ring_of_cliques():
    n, edges = ring_of_cliques(6, 5)
    rowptr, col = csr(n, edges)
    part, P = lv.louvain(n, rowptr, col)
    assert P == 6
    assert part == [i // 5 for i in range(n)]            # ids numbered by smallest member


def partitions(n):
    """All set partitions of range(n) as restricted-growth strings."""
    def rec(prefix, mx):
        if len(prefix) == n:
            yield prefix
            return
        for c in range(mx + 2):
            yield from rec(prefix + [c], max(mx, c))
    yield from rec([0], 0)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_louvain_against_brute_force_on_tiny_graphs(seed):
    """n = 8: the heuristic never beats the optimum over all 4140 partitions, is never worse
    than leaving every node alone, and its ids are in restricted-growth form."""
    rs = np.random.RandomState(seed)
    n = 8
    edges = hp.random_graph(n, 0.4, rs)
    if not edges:
        pytest.skip("empty graph")
    rowptr, col = csr(n, edges)
    part, P = lv.louvain(n, rowptr, col)
    q = lv.modularity(n, rowptr, col, part)
    best = max(lv.modularity(n, rowptr, col, pt) for pt in partitions(n))
    assert q <= best + 1e-12
    assert q >= lv.modularity(n, rowptr, col, list(range(n))) - 1e-12
    assert q >= 0.6 * best                                # a sane heuristic on these sizes
    seen = -1
    for c in part:
        assert c <= seen + 1
        seen = max(seen, c)
    assert P == seen + 1


def test_louvain_disconnected_cliques_and_empty_graph():
    """Disjoint cliques are exactly the communities (any merge lowers Q, any split too);
    a graph without edges keeps every node alone."""
    edges = []
    for c in range(4):
        for a, b in itertools.combinations(range(4), 2):
            edges.append((c * 4 + a, c * 4 + b))
    rowptr, col = csr(16, edges)
    part, P = lv.louvain(16, rowptr, col)
    assert P == 4 and part == [i // 4 for i in range(16)]
    rowptr0, col0 = csr(5, [])
    part0, P0 = lv.louvain(5, rowptr0, col0)
    assert P0 == 5 and part0 == list(range(5))


def test_louvain_levels_never_lower_modularity():
    rs = np.random.RandomState(9)
    n = 120
    edges = hp.random_graph(n, 0.05, rs)
    rowptr, col = csr(n, edges)
    q_prev = lv.modularity(n, rowptr, col, list(range(n)))
    for levels in (1, 2, 3, 32):
        part, _ = lv.louvain(n, rowptr, col, max_levels=levels)
        q = lv.modularity(n, rowptr, col, part)
        assert q >= q_prev - 1e-12
        q_prev = q
    assert q_prev > 0.2


def test_pack_parts_keeps_communities_whole_and_balances():
    """Pins: no community is split; at most max_parts groups; the heaviest group exceeds the
    lightest by at most the largest community (the greedy rule's bound); untouched when
    there are few enough communities; a worked case by hand."""
    rs = np.random.RandomState(3)
    part = rs.randint(0, 40, 500).tolist()
    part = [min(c, 39) for c in part]
    out, P = lv.pack_parts(part, 40, 6)
    assert P == 6 and set(out) <= set(range(6))
    for c in range(40):
        assert len({out[i] for i in range(500) if part[i] == c}) <= 1
    sizes = np.bincount(part, minlength=40)
    loads = np.bincount(out, minlength=6)
    assert loads.max() - loads.min() <= sizes.max()
    same, P2 = lv.pack_parts(part, 40, 64)
    assert same == part and P2 == 40
    # sizes 5,4,3,3,1 into 2 groups: 5->g0, 4->g1, 3->g1 (4<5), 3->g0 (5<7), 1->g1 (7<8)
    hand = [0] * 5 + [1] * 4 + [2] * 3 + [3] * 3 + [4]
    out2, _ = lv.pack_parts(hand, 5, 2)
    assert [out2[0], out2[5], out2[9], out2[12], out2[15]] == [0, 1, 1, 0, 1]
