"""gco_round_repair_static (the entry point that allocates nothing: its work area is a fixed
block inside the library's code object) against gco_round_repair, through the C ABI, bit for
bit: two calls in a row, the second on a smaller graph, so that whatever the first left in
the block must not show; then the size limit."""
import numpy as np
import pytest

from paper_2511_09261_amd import inputs

pytestmark = pytest.mark.gpu


def context_with_probabilities(gco, n, seed, problem="mis"):
    g = inputs.random_regular(n, 6, seed)
    P = 5
    part = inputs.bfs_partition(g, P, seed)
    E, Ws = inputs.init_params(g.n, part, P, 2, 16, seed)
    ctx = gco.Context(problem=problem, num_layers=2, dim=16)
    ctx.upload_graph(g.n, g.rowptr, g.col, part, P)
    ctx.set_params((E * 5).astype(np.float32), [W * 1.5 for W in Ws])
    ctx.forward()
    return ctx


def same_results(ctx):
    for scope in ("none", "local", "all"):
        want = ctx.round_repair(0.5, scope)
        got = ctx.round_repair_static(0.5, scope)
        np.testing.assert_array_equal(got[0], want[0])
        assert got[1:] == want[1:], scope
    x, size, before, after = ctx.round_repair_static(0.5, "all")
    return int(x.sum()), size, before, after


def test_static_work_area_gives_the_same_bits_twice_in_a_row(gco):
    big = context_with_probabilities(gco, 6001, seed=3)
    kept, size, before, after = same_results(big)
    assert kept == size > 0 and before > 0 and after == 0      # the repair had work to do
    small = context_with_probabilities(gco, 901, seed=4)
    kept, size, before, after = same_results(small)
    assert kept == size > 0 and before > 0 and after == 0
    # Max-Cut: no repair, the objective is the cut value
    cut = context_with_probabilities(gco, 1500, seed=5, problem="maxcut")
    same_results(cut)
    # and the larger graph once more, after the smaller ones
    same_results(big)
    for ctx in (big, small, cut):
        ctx.destroy()


def test_static_work_area_has_a_size_limit(gco):
    n = (1 << 21) + 1
    ctx = gco.Context(num_layers=1, dim=8)
    ctx.upload_graph(n, np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), None, 1)
    ctx.set_params(np.zeros((n, 8), dtype=np.float32), [np.zeros((1, 8, 1), dtype=np.float32)])
    ctx.forward()
    x, size, _, _ = ctx.round_repair(0.5, "local")               # p = 0.5 everywhere: all selected
    assert size == n
    with pytest.raises(gco.GcoError) as e:
        ctx.round_repair_static(0.5, "local")
    assert e.value.code == gco.ERANGE
    ctx.destroy()
    with pytest.raises(gco.GcoError) as e:                       # nothing to round yet
        gco.Context().round_repair_static(0.5, "none")
    assert e.value.code == gco.ESTATE
