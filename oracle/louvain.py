"""Checker for the graph partitioning step: modularity and the Louvain heuristic (Sec. 3.1).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing on the product path).  Plain
Python on dictionaries and integers, slow and meant to be read next to the paper.

Modularity of a partition of an undirected graph with m edges (unit weights; after an
aggregation step weights are edge counts):
    Q = sum over communities c of  in_c / m  -  (tot_c / 2m)^2
with in_c the weight of the edges inside c (each edge once) and tot_c the sum of the
degrees of c's nodes.  Putting an isolated node i (degree k_i, weight k_ic to the nodes of
c, tot_c taken without i) into community c changes Q by
    dQ = k_ic / m  -  tot_c k_i / (2 m^2)                                  (Sec. 3.1, Eq. 2)
which is Eq. 1 with the community's internal weight counted in both directions.  All
comparisons are made on the integer  2 m^2 dQ = 2 m k_ic - tot_c k_i,  so the procedure has
no rounding and two implementations agree id for id.

The heuristic, made deterministic:
  * level graph: nodes with integer edge weights and a self weight (edges inside the
    super-node, each once); the degree of a node is the sum of its edge weights plus twice
    its self weight;
  * local moving: nodes are visited in ascending id, sweep after sweep, until a sweep moves
    nothing; a node is taken out of its community, the gain of every neighbouring community
    and of its old one is computed, and it goes to the community of largest gain if that
    gain is strictly larger than the gain of going back; ties go to the smallest
    community id;
  * aggregation: communities become nodes, numbered by their smallest member; the levels
    end when a level moves nothing (or after max_levels levels).
Final community ids are numbered by smallest original member.
"""
from __future__ import annotations


def modularity(n, rowptr, col, part):
    """Q by its definition, in Python floats (fp64)."""
    m2 = int(rowptr[n])  # 2m
    if m2 == 0:
        return 0.0
    inside = {}
    tot = {}
    for i in range(n):
        c = int(part[i])
        tot[c] = tot.get(c, 0) + int(rowptr[i + 1] - rowptr[i])
        for e in range(int(rowptr[i]), int(rowptr[i + 1])):
            if int(part[int(col[e])]) == c:
                inside[c] = inside.get(c, 0) + 1  # both directions: twice the inside weight
    q = 0.0
    for c, t in tot.items():
        q += inside.get(c, 0) / m2 - (t / m2) ** 2
    return q


def gain_times_2m2(m, k_ic, tot_c, k_i):
    """2 m^2 dQ of Eq. 2, an integer."""
    return 2 * m * k_ic - tot_c * k_i


def _local_moving(adj, self_w, m):
    """adj[i] = {j: w}; returns (community of every node, whether anything moved)."""
    N = len(adj)
    k = [sum(adj[i].values()) + 2 * self_w[i] for i in range(N)]
    comm = list(range(N))
    tot = k[:]
    moved_any = False
    while True:
        moved = False
        for i in range(N):
            old = comm[i]
            w_to = {}
            for j, w in adj[i].items():
                w_to[comm[j]] = w_to.get(comm[j], 0) + w
            tot[old] -= k[i]
            stay = gain_times_2m2(m, w_to.get(old, 0), tot[old], k[i])
            best_c, best_g = old, stay
            for c in sorted(w_to):
                g = gain_times_2m2(m, w_to[c], tot[c], k[i])
                if g > best_g:
                    best_c, best_g = c, g
            comm[i] = best_c
            tot[best_c] += k[i]
            if best_c != old:
                moved = True
        if not moved:
            break
        moved_any = True
    return comm, moved_any


def louvain(n, rowptr, col, max_levels=32):
    """Community id of every node (ids numbered by smallest member) and the number of
    communities."""
    m = int(rowptr[n]) // 2
    member_of = list(range(n))           # original node -> node of the current level
    adj = [dict() for _ in range(n)]
    for i in range(n):
        for e in range(int(rowptr[i]), int(rowptr[i + 1])):
            adj[i][int(col[e])] = 1
    self_w = [0] * n
    if m > 0:
        for _ in range(max_levels):
            comm, moved = _local_moving(adj, self_w, m)
            if not moved:
                break
            # number the communities by their smallest member
            new_id = {}
            for i in range(len(adj)):
                if comm[i] not in new_id:
                    new_id[comm[i]] = len(new_id)
            N2 = len(new_id)
            adj2 = [dict() for _ in range(N2)]
            self2 = [0] * N2
            for i in range(len(adj)):
                a = new_id[comm[i]]
                self2[a] += self_w[i]
                for j, w in adj[i].items():
                    b = new_id[comm[j]]
                    if a == b:
                        if i < j:
                            self2[a] += w
                    else:
                        adj2[a][b] = adj2[a].get(b, 0) + w
            member_of = [new_id[comm[x]] for x in member_of]
            adj, self_w = adj2, self2
    # final ids by smallest original member
    final = {}
    part = [0] * n
    for i in range(n):
        c = member_of[i]
        if c not in final:
            final[c] = len(final)
        part[i] = final[c]
    return part, len(final)


def pack_parts(part, num_parts, max_parts):
    """Merge communities into at most max_parts groups without splitting any (merging never
    cuts an edge): communities in the order (size descending, id ascending), each to the
    group with the fewest nodes so far (ties: smallest group id).  Returns the group of every
    node and the number of groups; with num_parts <= max_parts nothing changes."""
    n = len(part)
    if num_parts <= max_parts:
        return list(part), num_parts
    size = [0] * num_parts
    for c in part:
        size[c] += 1
    order = sorted(range(num_parts), key=lambda c: (-size[c], c))
    load = [0] * max_parts
    group = [0] * num_parts
    for c in order:
        b = min(range(max_parts), key=lambda x: (load[x], x))
        group[c] = b
        load[b] += size[c]
    return [group[c] for c in part], max_parts
