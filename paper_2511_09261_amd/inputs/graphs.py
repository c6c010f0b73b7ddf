"""Seeded synthetic graphs, partition ids and initial parameters.

These stand in for the paper's inputs (Sec. 4.1.3: regular graphs of a chosen
degree; SNAP social networks of which only node count, edge count and degree
shape are taken, Tables 1 and 2).  Everything is made from the counter-based
streams of ``rng`` and returned as plain numpy arrays that both the checker and
the device library consume.  No arithmetic of the training method lives here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from . import rng

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbfs_partition.so")
_lib = None


def build_native(force: bool = False) -> str:
    """Compile the BFS partitioner with gcc (about a second)."""
    src = os.path.join(_HERE, "bfs_partition.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", src, "-o", _LIB_PATH])
    return _LIB_PATH


def _native():
    global _lib
    if _lib is None:
        build_native()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.bfs_region_growing.restype = ctypes.c_int
        _lib.bfs_region_growing.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    return _lib


@dataclass
class Graph:
    """Simple undirected graph as a symmetric CSR with ascending columns."""
    n: int
    rowptr: np.ndarray  # int64 [n+1]
    col: np.ndarray     # int32 [2m]

    @property
    def m(self) -> int:
        return int(self.col.shape[0] // 2)

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr)

    def edges(self) -> np.ndarray:
        """[m, 2] int64 array of (u, v) with u < v, sorted."""
        row = np.repeat(np.arange(self.n, dtype=np.int64), np.diff(self.rowptr))
        c = self.col.astype(np.int64)
        keep = row < c
        return np.stack([row[keep], c[keep]], axis=1)


def from_edges(n: int, u: np.ndarray, v: np.ndarray) -> Graph:
    """Canonicalise an edge list: drop loops and duplicates, symmetrise, sort."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    keep = u != v
    u, v = u[keep], v[keep]
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    key = np.unique(lo * np.int64(n) + hi)
    lo, hi = key // n, key % n
    both = np.concatenate([lo * np.int64(n) + hi, hi * np.int64(n) + lo])
    both.sort()
    row, col = both // n, both % n
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=n), out=rowptr[1:])
    return Graph(n, rowptr, col.astype(np.int32))


def erdos_renyi(n: int, p: float, seed: int) -> Graph:
    """G(n, p): every pair i < j independently with probability p."""
    iu, ju = np.triu_indices(n, k=1)
    r = rng.uniform(rng.stream_key(seed, 1), iu.shape[0])
    keep = r < p
    return from_edges(n, iu[keep], ju[keep])


def random_regular(n: int, d: int, seed: int) -> Graph:
    """Configuration model: shuffle the n*d stubs and pair neighbours in the
    shuffled order; loops and repeated pairs are dropped, so a few nodes end
    with degree below d (expected count is O(d^2), independent of n)."""
    if (n * d) % 2:
        raise ValueError("n*d must be even")
    keys = rng.u64(rng.stream_key(seed, 2), n * d)
    order = np.argsort(keys, kind="stable")
    del keys
    stubs = (order // d).astype(np.int64)
    del order
    return from_edges(n, stubs[0::2], stubs[1::2])


def chung_lu_weights(n: int, m_target: int, gamma: float, w_max: float) -> np.ndarray:
    """w_i = w_max * ((i + 1 + i0) / (1 + i0)) ** (-1 / (gamma - 1)), with i0
    chosen by bisection so that sum(w) = 2 * m_target."""
    a = 1.0 / (gamma - 1.0)
    i = np.arange(n, dtype=np.float64)

    def total(i0):
        return float(np.sum(w_max * ((i + 1.0 + i0) / (1.0 + i0)) ** (-a)))

    lo, hi = 0.0, 1.0
    while total(hi) < 2.0 * m_target and hi < 1e12:
        hi *= 2.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if total(mid) < 2.0 * m_target:
            lo = mid
        else:
            hi = mid
    i0 = 0.5 * (lo + hi)
    return w_max * ((i + 1.0 + i0) / (1.0 + i0)) ** (-a)


def chung_lu(n: int, m_target: int, gamma: float, w_max: float, seed: int,
             rounds: int = 8) -> Graph:
    """Power-law graph: endpoint pairs drawn i.i.d. proportional to the weights.

    Pairs are drawn in rounds; each round draws as many pairs as are still
    missing after loops and duplicates are removed, so the realised m ends
    close to (never above) m_target.  Node labels are then shuffled so that
    the heavy rows are scattered over the id range as in a real data set.
    """
    w = chung_lu_weights(n, m_target, gamma, w_max)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    keys = np.empty(0, dtype=np.int64)
    drawn = 0
    for _ in range(rounds):
        need = m_target - keys.shape[0]
        if need <= 0:
            break
        r = rng.uniform(rng.stream_key(seed, 3), 2 * need, offset=2 * drawn)
        drawn += need
        ends = np.minimum(np.searchsorted(cdf, r, side="right"), n - 1).astype(np.int64)
        a, b = ends[0::2], ends[1::2]
        ok = a != b
        lo, hi = np.minimum(a[ok], b[ok]), np.maximum(a[ok], b[ok])
        keys = np.unique(np.concatenate([keys, lo * np.int64(n) + hi]))
    relabel = np.argsort(rng.u64(rng.stream_key(seed, 4), n), kind="stable").astype(np.int64)
    return from_edges(n, relabel[keys // n], relabel[keys % n])


def bfs_partition(g: Graph, num_parts: int, seed: int) -> np.ndarray:
    """part_id int32[n] from seeded BFS region growing (see bfs_partition.c)."""
    n = g.n
    if num_parts == 1:
        return np.zeros(n, dtype=np.int32)
    roots, seen, off = [], set(), 0
    key = rng.stream_key(seed, 5)
    while len(roots) < num_parts:
        for c in rng.below(key, num_parts, n, offset=off):
            c = int(c)
            if c not in seen and len(roots) < num_parts:
                seen.add(c)
                roots.append(c)
        off += num_parts
    roots = np.asarray(roots, dtype=np.int32)
    part = np.empty(n, dtype=np.int32)
    rp = np.ascontiguousarray(g.rowptr, dtype=np.int64)
    cl = np.ascontiguousarray(g.col, dtype=np.int32)
    rc = _native().bfs_region_growing(n, rp.ctypes.data, cl.ctypes.data, num_parts,
                                      roots.ctypes.data, part.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"bfs_region_growing failed: {rc}")
    return part


def init_params(n: int, part: np.ndarray, num_parts_w: int, num_layers: int,
                dim: int, seed: int):
    """Initial parameters as float32 arrays.

    E[i, :] ~ N(0, 0.1^2), drawn from a stream indexed by the ORIGINAL node id, so
    a node's embedding does not depend on how the graph is partitioned.
    W_l[k] ~ U(-a, a), a = sqrt(6 / (d_in + d_out)), one stream per (layer,
    partition).  Returns (E [n, dim], [W_1 .. W_L]) with W_l of shape
    [num_parts_w, dim, dim] for l < L and [num_parts_w, dim, 1] for l = L.
    """
    del part
    E = (0.1 * rng.normal(rng.stream_key(seed, 10), n * dim)).astype(np.float32).reshape(n, dim)
    Ws = []
    for l in range(1, num_layers + 1):
        d_out = dim if l < num_layers else 1
        a = np.sqrt(6.0 / (dim + d_out))
        W = np.empty((num_parts_w, dim, d_out), dtype=np.float32)
        for k in range(num_parts_w):
            u = rng.uniform(rng.stream_key(seed, 11, l, k), dim * d_out)
            W[k] = ((2.0 * u - 1.0) * a).astype(np.float32).reshape(dim, d_out)
        Ws.append(W)
    return E, Ws


def gumbel_uniforms(n: int, dim: int, seed: int) -> np.ndarray:
    """float32 uniforms strictly inside (0, 1), one per embedding element, from a stream
    indexed by the ORIGINAL node id: the noise source of the Gumbel-softmax input
    processing (23 random bits, offset by half a step: every value is an exact float32 in
    [2^-24, 1 - 2^-24])."""
    k = rng.u64(rng.stream_key(seed, 12), n * dim) >> np.uint64(41)
    return ((k.astype(np.float64) + 0.5) / float(1 << 23)).astype(np.float32).reshape(n, dim)


def exploration_uniforms(rounds: int, seed: int) -> np.ndarray:
    """float64 uniforms in [0, 1), two per round: the random draws of the cross-subgraph
    coordination stage's epsilon-greedy agent (explore or not; which option)."""
    return rng.uniform(rng.stream_key(seed, 13), 2 * rounds).reshape(rounds, 2)


# --- the five workload configurations ---------------------------------------

@dataclass
class Workload:
    name: str
    problem: str          # "mis" | "maxcut"
    graph: Graph
    part: np.ndarray      # int32 [n]
    num_parts: int
    num_layers: int
    dim: int
    storage: str          # "fp32" | "bf16"
    lr: float
    epochs: int
    seed: int


def make_workload(name: str, scale: float = 1.0) -> Workload:
    """Build one of the configured workloads.  ``scale`` < 1 shrinks node and
    edge counts proportionally (partition count kept) for quick checks."""
    if name == "c1":
        g = erdos_renyi(200, 0.05, seed=0)
        return Workload(name, "mis", g, bfs_partition(g, 1, 0), 1, 2, 16, "fp32", 1e-2, 200, 0)
    if name == "c2":
        n = max(8 * 8, int(10_000 * scale) // 2 * 2)
        g = random_regular(n, 3, seed=1)
        return Workload(name, "maxcut", g, bfs_partition(g, 8, 1), 8, 2, 32, "fp32", 1e-2, 500, 1)
    if name == "c3":
        n, m = int(4_039 * scale), int(88_234 * scale)
        g = chung_lu(n, m, 2.5, 1_000.0 * min(1.0, scale ** 0.5), seed=2)
        return Workload(name, "mis", g, bfs_partition(g, 16, 2), 16, 2, 64, "bf16", 5e-3, 300, 2)
    if name in ("c4", "c4p1"):
        n, m = int(1_134_890 * scale), int(2_987_624 * scale)
        g = chung_lu(n, m, 2.2, 28_000.0 * min(1.0, scale ** 0.5), seed=3)
        P = 64 if name == "c4" else 1
        return Workload(name, "mis", g, bfs_partition(g, P, 3), P, 3, 64, "bf16", 5e-3, 100, 3)
    if name in ("c5", "c5p1"):
        n = int(2_000_000 * scale) // 2 * 2
        g = random_regular(n, 50, seed=4)
        P = 256 if name == "c5" else 1
        return Workload(name, "maxcut", g, bfs_partition(g, P, 4), P, 3, 128, "bf16", 5e-3, 50, 4)
    raise ValueError(f"unknown workload {name!r}")


def describe(wl: Workload) -> dict:
    """Realised structure of a workload, printed next to every measurement."""
    g, part = wl.graph, wl.part
    e = g.edges()
    local = part[e[:, 0]] == part[e[:, 1]]
    row = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    loc_entry = part[row] == part[g.col]
    ldeg = np.bincount(row[loc_entry], minlength=g.n)
    sizes = np.bincount(part, minlength=wl.num_parts)
    return {
        "name": wl.name, "n": g.n, "m": g.m, "P": wl.num_parts,
        "m_local": int(local.sum()), "m_cut": int((~local).sum()),
        "max_degree": int(g.degrees().max(initial=0)),
        "max_local_degree": int(ldeg.max(initial=0)),
        "locally_isolated": int((ldeg == 0).sum()),
        "part_size_min": int(sizes.min()), "part_size_max": int(sizes.max()),
    }
