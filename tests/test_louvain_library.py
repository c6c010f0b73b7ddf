"""The library's partitioner (gco_louvain, host code) against the checker: the procedure is
deterministic and compares exact integers, so community ids agree one by one."""
import numpy as np
import pytest

from oracle import louvain as lv
from paper_2511_09261_amd import binding, inputs
from tests import helpers as hp


def _lib_or_skip():
    try:
        binding.load()
    except OSError as e:           # not built
        pytest.skip(str(e))


@pytest.mark.parametrize("n,p,seed", [(60, 0.1, 0), (200, 0.03, 1), (500, 0.01, 2), (37, 0.0, 3)])
def test_ids_equal_the_checker_on_random_graphs(n, p, seed):
    _lib_or_skip()
    rs = np.random.RandomState(seed)
    edges = hp.random_graph(n, p, rs)
    rowptr, col = hp.csr_from_edges(n, edges)
    part, P, q = binding.louvain(n, rowptr, col)
    want, wantP = lv.louvain(n, rowptr, col)
    assert P == wantP
    np.testing.assert_array_equal(part, want)
    assert q == pytest.approx(lv.modularity(n, rowptr, col, want), abs=1e-12)


@pytest.mark.parametrize("levels", [0, 1, 2])
def test_level_limit_and_power_law_graph(levels):
    """A scaled-down c3-shaped graph (power-law degrees, a few hubs), stopped early too."""
    _lib_or_skip()
    g = inputs.chung_lu(1200, 9000, 2.5, 300.0, seed=7)
    part, P, q = binding.louvain(g.n, g.rowptr, g.col, max_levels=levels)
    want, wantP = lv.louvain(g.n, g.rowptr, g.col, max_levels=levels)
    np.testing.assert_array_equal(part, want)
    assert P == wantP
    if levels == 0:
        assert P == g.n


def test_malformed_graphs_are_refused():
    _lib_or_skip()
    rowptr = np.array([0, 1, 2], dtype=np.int64)
    with pytest.raises(binding.GcoError):
        binding.louvain(2, rowptr, np.array([0, 0], dtype=np.int32))       # self loop
    with pytest.raises(binding.GcoError):
        binding.louvain(2, rowptr, np.array([1, 5], dtype=np.int32))       # column out of range
    with pytest.raises(binding.GcoError):
        binding.louvain(2, np.array([0, 1, 1], dtype=np.int64), np.array([1], dtype=np.int32))  # odd


@pytest.mark.parametrize("max_parts", [1, 7, 64, 1000])
def test_pack_parts_equals_the_checker(max_parts):
    _lib_or_skip()
    g = inputs.chung_lu(3000, 6000, 2.3, 200.0, seed=11)
    part, P, _ = binding.louvain(g.n, g.rowptr, g.col)
    got, gotP = binding.pack_parts(part, P, max_parts)
    want, wantP = lv.pack_parts(part.tolist(), P, max_parts)
    assert gotP == wantP
    np.testing.assert_array_equal(got, want)
    with pytest.raises(binding.GcoError):
        binding.pack_parts(np.array([0, 3], dtype=np.int32), 2, 1)
