"""The seeded input generators: structure, determinism, balance (CPU only)."""
import numpy as np
import pytest

from paper_2511_09261_amd import inputs
from paper_2511_09261_amd.inputs import rng


def check_simple_symmetric(g):
    assert g.rowptr[0] == 0 and g.rowptr[-1] == g.col.shape[0]
    row = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    col = g.col.astype(np.int64)
    assert (row != col).all()
    key = row * g.n + col
    assert (np.diff(key) > 0).all()                  # sorted rows, no duplicates
    assert np.array_equal(np.sort(col * g.n + row), key)   # symmetric


def test_splitmix64_reference_values():
    """First outputs of SplitMix64 seeded with 0 (Steele, Lea, Flood 2014;
    the constants are those of the published generator)."""
    out = rng.u64(0, 3)
    assert [int(v) for v in out] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    # slices of a stream are reproducible
    a = rng.u64(123, 1000)
    assert np.array_equal(a[100:200], rng.u64(123, 100, offset=100))
    z = rng.normal(5, 50)
    assert np.array_equal(z[10:20], rng.normal(5, 10, offset=10))


@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
def test_workloads_are_simple_symmetric_and_deterministic(name):
    a = inputs.make_workload(name)
    b = inputs.make_workload(name)
    check_simple_symmetric(a.graph)
    assert np.array_equal(a.graph.col, b.graph.col) and np.array_equal(a.part, b.part)
    sizes = np.bincount(a.part, minlength=a.num_parts)
    cap = -(-a.graph.n // a.num_parts)
    assert sizes.max() <= cap and sizes.sum() == a.graph.n and a.part.min() >= 0
    d = inputs.describe(a)
    assert d["m_local"] + d["m_cut"] == d["m"]


def test_shapes_of_the_small_workloads():
    c1 = inputs.describe(inputs.make_workload("c1"))
    assert c1["n"] == 200 and 850 < c1["m"] < 1150 and c1["m_cut"] == 0
    c2 = inputs.make_workload("c2")
    deg = c2.graph.degrees()
    assert c2.graph.n == 10_000 and deg.max() == 3 and (deg == 3).mean() > 0.99
    c3 = inputs.describe(inputs.make_workload("c3"))
    assert c3["n"] == 4039 and 0.95 * 88_234 < c3["m"] <= 88_234 and c3["max_degree"] > 300


def test_power_law_graph_scaled_down():
    wl = inputs.make_workload("c4", scale=0.02)
    check_simple_symmetric(wl.graph)
    deg = wl.graph.degrees()
    assert deg.max() > 50 * np.median(deg[deg > 0])       # heavy tail
    assert (deg == 0).mean() > 0.05                        # isolated nodes exist
    sizes = np.bincount(wl.part, minlength=64)
    assert sizes.max() - sizes.min() <= 1


def test_bfs_regions_are_connected_where_the_graph_allows():
    g = inputs.random_regular(2000, 4, seed=9)
    part = inputs.bfs_partition(g, 4, seed=9)
    e = g.edges()
    # region growing keeps far more edges inside regions than a random split would (1/4)
    assert (part[e[:, 0]] == part[e[:, 1]]).mean() > 0.5


def test_parameters_do_not_depend_on_the_partition():
    E1, W1 = inputs.init_params(100, None, 3, 2, 8, seed=5)
    E2, W2 = inputs.init_params(100, None, 1, 2, 8, seed=5)
    assert np.array_equal(E1, E2) and np.array_equal(W1[0][0], W2[0][0])
    assert E1.dtype == np.float32 and W1[1].shape == (3, 8, 1)
    assert abs(E1.std() - 0.1) < 0.01 and np.abs(W1[0]).max() <= np.sqrt(6 / 16)
