"""The checker's cross-subgraph coordination stage (oracle/coordinate.py, CPU only).

The stage follows one reading of Sec. 3.3 / Alg. 1 stage 3 (parity unpinned: the paper
fixes neither state, reward nor schedule).  What can be fixed is fixed here: the score is
the pinned loss evaluated on 0/1 vectors of the whole graph; the base action is a cover of
the conflict edges built by the stated rule (hand example); the run keeps the best
assignment, never ends worse than it starts, stops when no conflict is left, and is a
function of its inputs alone."""
import numpy as np
import pytest

from oracle import combinatorial as cb
from oracle import coordinate as co
from oracle import gcn
from paper_2511_09261_amd import inputs
from tests import helpers as hp


def test_score_is_minus_the_loss_of_the_whole_graph_on_a_bitstring():
    rs = np.random.RandomState(0)
    n = 40
    rowptr, col = hp.csr_from_edges(n, hp.random_graph(n, 0.15, rs))
    whole = gcn.local_graph(n, rowptr, col, None, 1, "sym")
    for _ in range(10):
        x = (rs.random(n) < 0.5).astype(np.uint8)
        for a, b in ((2.0, 1.0), (3.5, 0.5)):
            want, _ = gcn.loss(whole, x.astype(np.float64), gcn.Spec(problem="mis", alpha=a, beta=b))
            assert co.score(n, rowptr, col, x, a, b) == pytest.approx(-want, abs=1e-12)


def test_linear_cover_by_hand():
    """Conflict edges (0,5) (0,7) (2,5) (3,9) with p = .9 .. .6 .8 .. .7 .. .55 .. .6:
    (0,5): p5 < p0 -> 5;  (0,7): neither chosen, p7 < p0 -> 7;  (2,5): covered by 5;
    (3,9): tie in p -> smaller id 3."""
    p = np.zeros(10, dtype=np.float32)
    p[[0, 2, 3, 5, 7, 9]] = [0.9, 0.6, 0.6, 0.7, 0.55, 0.6]
    cu, cv = np.array([0, 0, 2, 3]), np.array([5, 7, 5, 9])
    chosen, at, other = co.linear_cover(cu, cv, p)
    assert chosen == [5, 7, 3] and at == [0, 1, 3] and other == [0, 0, 9]
    # forcing the other end at the first edge: 0 is taken, which also covers (0,7); (2,5) now chooses
    chosen, at, other = co.linear_cover(cu, cv, p, forced=0)
    assert chosen == [0, 2, 3] and at == [0, 2, 3] and other == [5, 5, 9]
    # forcing an edge at which no choice is made changes nothing
    assert co.linear_cover(cu, cv, p, forced=2)[0] == [5, 7, 3]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cover_covers_every_conflict_with_its_own_ends(seed):
    rs = np.random.RandomState(seed)
    m = 60
    cu = rs.randint(0, 30, m)
    cv = cu + 1 + rs.randint(0, 30, m)
    order = np.lexsort((cv, cu))
    cu, cv = cu[order], cv[order]
    p = rs.random(70).astype(np.float32)
    for forced in (-1, 0, 7, 31):
        chosen, at, other = co.linear_cover(cu, cv, p, forced)
        s = set(chosen)
        assert len(s) == len(chosen)
        assert all(int(u) in s or int(v) in s for u, v in zip(cu, cv))
        for node, e, o in zip(chosen, at, other):
            assert {node, o} == {int(cu[e]), int(cv[e])}


def trained_case(seed, epochs=60):
    g = inputs.random_regular(240, 4, seed)
    P = 4
    part = inputs.bfs_partition(g, P, seed)
    E, Ws = inputs.init_params(g.n, part, P, 2, 16, seed)
    spec = gcn.Spec(problem="mis", num_layers=2, lr=2e-2)
    lg = gcn.local_graph(g.n, g.rowptr, g.col, part, P, "sym")
    st = gcn.init_state(E, Ws)
    gcn.train(lg, st, spec, epochs)
    return g, part, P, lg, st, spec


def test_the_stage_keeps_the_best_and_is_a_function_of_its_inputs():
    g, part, P, lg, st, spec = trained_case(3)
    rl = co.RLSpec(rounds=8, epochs=6, lam=1.5, epsilon=0.5)
    U = inputs.exploration_uniforms(rl.rounds, 5)
    import copy
    out = co.coordinate(g.n, g.rowptr, g.col, part, lg, copy.deepcopy(st), spec, rl, U)
    again = co.coordinate(g.n, g.rowptr, g.col, part, lg, copy.deepcopy(st), spec, rl, U)
    assert out["actions"] == again["actions"] and out["scores"] == again["scores"]
    np.testing.assert_array_equal(out["x_best"], again["x_best"])
    assert out["conflicts"][0] > 0                                   # there was something to coordinate
    assert len(out["scores"]) == len(out["actions"]) + 1
    assert out["score_best"] == max(out["scores"]) >= out["scores"][0]
    assert co.score(g.n, g.rowptr, g.col, out["x_best"], spec.alpha, spec.beta) == out["score_best"]
    # the penalised nodes of a round are ends of that round's conflicts, one subgraph each
    cut_u, cut_v = cb.cut_edges_vectorised(g.n, g.rowptr, g.col, part)
    assert all(len(c) > 0 for c in out["chosen"])
    # penalties push the chosen nodes down: fewer cross conflicts at the end than at the start
    assert min(out["conflicts"]) < out["conflicts"][0]
    # some exploration happened and brought a node in
    assert any(a >= 0 for a in out["actions"])


def test_greedy_agent_without_exploration_takes_the_base_action_first():
    g, part, P, lg, st, spec = trained_case(4)
    rl = co.RLSpec(rounds=3, epochs=4, epsilon=0.0)
    out = co.coordinate(g.n, g.rowptr, g.col, part, lg, st, spec, rl, np.zeros((3, 2)))
    assert out["actions"][0] == -1                                   # all Q are 0: first candidate
    assert set(k[1] for k in out["Q"]) <= set(out["actions"])


def test_no_cross_edge_means_no_round():
    g, part, P, lg, st, spec = trained_case(5, epochs=0)
    whole = gcn.local_graph(g.n, g.rowptr, g.col, None, 1, "sym")
    one = gcn.init_state(st.E, [W[:1] for W in st.Ws])
    out = co.coordinate(g.n, g.rowptr, g.col, np.zeros(g.n, dtype=np.int32), whole, one, spec,
                        co.RLSpec(rounds=4), np.zeros((4, 2)))
    assert out["actions"] == [] and out["conflicts"] == [0] and len(out["scores"]) == 1
