"""GPU parity on the configured workloads, at their full sizes and in the launch
configuration the benchmark times.

  c1, c2 (fp32)  ten-epoch loss trajectory within 1e-4; after the configured number
                 of epochs the objective is within 1 % of the checker's and the
                 repaired solution is feasible on both sides
  c3, c4 (bf16)  probabilities, hidden activations and gradients at the initial
                 weights within 2e-2 (tests/parity.py: every ReLU decision the checker
                 can settle must be the checker's, gradient entries get the slack of the
                 undecidable units that reach them); ten-epoch loss trajectory within
                 2e-2; integer read-out bit-exact on the device's own probabilities
  c5 (bf16)      the same at fixed weights on a seeded sample of subgraphs, each
                 run through the checker alone (subgraphs are independent)
"""
import dataclasses

import numpy as np
import pytest

from oracle import combinatorial as cb
from oracle import gcn
from paper_2511_09261_amd import inputs
from tests import parity
from tests.parity import rel, rel_l2

pytestmark = pytest.mark.gpu


def setup(gco, wl):
    g = wl.graph
    E, Ws = inputs.init_params(g.n, wl.part, wl.num_parts, wl.num_layers, wl.dim, wl.seed)
    ctx = gco.Context(problem=wl.problem, num_layers=wl.num_layers, dim=wl.dim,
                      storage=wl.storage, lr=wl.lr)
    ctx.upload_graph(g.n, g.rowptr, g.col, wl.part, wl.num_parts)
    ctx.set_params(E, Ws)
    bf16 = wl.storage == "bf16"
    spec = gcn.Spec(problem=wl.problem, num_layers=wl.num_layers, lr=wl.lr,
                    storage="bf16" if bf16 else "exact")
    lg = gcn.local_graph(g.n, g.rowptr, g.col, wl.part, wl.num_parts, "sym")
    return ctx, spec, lg, E, Ws


def check_readout(ctx, wl, scope="local"):
    """Rounding, repair, cross edges on the device's own probabilities: bit-exact."""
    g = wl.graph
    ctx.forward()
    p = ctx.get_probs()
    x0, _, cb0, _ = ctx.round_repair(0.5, "none")
    np.testing.assert_array_equal(x0, cb.round_probs(p))
    assert cb0 == cb.count_conflicts(g.n, g.rowptr, g.col, wl.part, x0, "all")
    x, obj, _, cafter = ctx.round_repair(0.5, scope)
    if wl.problem == "mis":
        want = cb.repair(g.n, g.rowptr, g.col, wl.part, p, x0, scope)
        np.testing.assert_array_equal(x, want)
        assert obj == want.sum()
        assert cb.count_conflicts(g.n, g.rowptr, g.col, wl.part, x, scope) == 0
    else:
        np.testing.assert_array_equal(x, x0)
        assert obj == cb.cut_value(g.n, g.rowptr, g.col, wl.part, x, "all")
    assert cafter == cb.count_conflicts(g.n, g.rowptr, g.col, wl.part, x, "all")
    u, v = ctx.cut_edges()
    wu, wv = cb.cut_edges_vectorised(g.n, g.rowptr, g.col, wl.part)
    np.testing.assert_array_equal(u, wu)
    np.testing.assert_array_equal(v, wv)
    np.testing.assert_array_equal(ctx.cross_mask(), cb.cross_mask(g.n, wu, wv))
    return p, x, obj


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_fp32_workloads_full_training(gco, name):
    wl = inputs.make_workload(name)
    ctx, spec, lg, E, Ws = setup(gco, wl)
    got = ctx.train(wl.epochs)
    st = gcn.init_state(E, Ws)
    want, _ = gcn.train(lg, st, spec, wl.epochs)
    assert np.abs(got[:10] - want[:10]).max() <= 1e-4 * np.abs(want[:10]).max()
    # end of training: objective within 1 %, same feasibility after repair
    g = wl.graph
    p_dev, x_dev, obj_dev = check_readout(ctx, wl)
    p_ref = gcn.forward(lg, st.E, st.Ws, spec)["p"].astype(np.float32)
    tot_dev, _ = ctx.loss()
    tot_ref, _ = gcn.loss(lg, p_ref.astype(np.float64), spec)
    assert abs(tot_dev - tot_ref) <= 1e-2 * abs(tot_ref)
    x_ref = cb.round_probs(p_ref)
    if wl.problem == "mis":
        x_ref = cb.repair(g.n, g.rowptr, g.col, wl.part, p_ref, x_ref, "local")
        obj_ref = int(x_ref.sum())
        feas_ref = cb.count_conflicts(g.n, g.rowptr, g.col, wl.part, x_ref, "local") == 0
        feas_dev = cb.count_conflicts(g.n, g.rowptr, g.col, wl.part, x_dev, "local") == 0
        assert feas_ref and feas_dev
    else:
        obj_ref = cb.cut_value(g.n, g.rowptr, g.col, wl.part, x_ref, "all")
    assert abs(obj_dev - obj_ref) <= max(1, 1e-2 * abs(obj_ref))
    ctx.destroy()


def fixed_weight_checks(ctx, spec, lg, E, Ws, label, plain=False):
    parity.compare_bf16_run(ctx, lg, E, Ws, spec, label=label, plain=plain)


def test_c3_bf16_workload(gco):
    wl = inputs.make_workload("c3")
    ctx, spec, lg, E, Ws = setup(gco, wl)
    fixed_weight_checks(ctx, spec, lg, E, Ws, "c3")
    got = ctx.train(10)
    st = gcn.init_state(E, Ws)
    want, _ = gcn.train(lg, st, spec, 10)
    assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
    ctx.train(wl.epochs - 10, return_loss=False)
    gcn.train(lg, st, spec, wl.epochs - 10)
    tot_dev, _ = ctx.loss()
    tot_ref, _ = gcn.loss(lg, gcn.forward(lg, st.E, st.Ws, spec)["p"], spec)
    assert abs(tot_dev - tot_ref) <= 1e-2 * abs(tot_ref)
    check_readout(ctx, wl, "local")
    check_readout(ctx, wl, "all")
    ctx.destroy()


C4_SAMPLE = (3, 17, 40, 63)


@pytest.mark.timeout(1200)
def test_c4_youtube_shaped_full_size(gco):
    """The benchmark's workload (1.13 M nodes, 64 subgraphs, 3 layers, width 64, bf16):
    fixed-weight comparison and ten-epoch trajectory against the checker on the whole
    batch, then the configured 100 epochs against the checker on four sampled subgraphs,
    each trained alone (subgraphs are independent: Sec. 3.3)."""
    wl = inputs.make_workload("c4")
    print("c4", inputs.describe(wl), flush=True)
    g = wl.graph
    ctx, spec, lg, E, Ws = setup(gco, wl)
    # at the workload's own initialisation the undecidable units carry so little gradient
    # that every entry also matches within 2e-2 without any slack
    fixed_weight_checks(ctx, spec, lg, E, Ws, "c4", plain=True)
    print("c4 fixed-weight checks done", flush=True)
    got = ctx.train(10)
    st = gcn.init_state(E, Ws)
    want = []
    for e in range(10):
        w, _ = gcn.train(lg, st, spec, 1)
        want.append(w[0])
        print(f"c4 checker epoch {e}: {w[0]:.3f} device {got[e]:.3f}", flush=True)
    want = np.array(want)
    assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
    # the loss falls by tens of thousands per epoch here, so the bound above is slack; every
    # epoch's value must also sit within 2e-2 of the smallest step the checker's loss takes
    assert np.abs(got - want).max() <= 2e-2 * np.abs(np.diff(want)).min()
    del st
    # deterministic: the same ten epochs again give the same bits
    ctx.set_params(E, Ws)
    np.testing.assert_array_equal(ctx.train(10), got)
    # end of training: the configured number of epochs
    ctx.train(wl.epochs - 10, return_loss=False)
    _, per_dev = ctx.loss()
    p_dev, x_dev, _ = check_readout(ctx, wl, "local")
    # A hundred epochs amplify rounding: where a hub's probability tips over, two correct
    # runs end in different local minima of that subgraph.  Measured on the device itself:
    # the same arithmetic with the scalar layer's fp32 sums taken in another order (two of
    # its launch forms) ends within 1.5e-6 of the same loss in the median subgraph, but 0.5 to
    # 2.7 % apart in 5 of the 64, while the loss of the whole graph differs by 8e-5.  The
    # checker shows which subgraphs are of that kind: it trains each sampled one with and
    # without the bf16 roundings.  Where those two agree to 1e-3 the device must match within
    # 1 %; elsewhere within 5 %; the sum over the sampled subgraphs within 1 %.
    import dataclasses
    spec_exact = dataclasses.replace(spec, storage="exact")
    sum_ref = sum_dev = 0.0
    for k in C4_SAMPLE:
        idx, sub = subgraph_alone(wl, k)
        lgk = gcn.local_graph(sub.n, sub.rowptr, sub.col, None, 1, "sym")
        stk = gcn.init_state(E[idx], [W[k:k + 1] for W in Ws])
        gcn.train(lgk, stk, spec, wl.epochs)
        p_ref = gcn.forward(lgk, stk.E, stk.Ws, spec)["p"]
        tot_ref, _ = gcn.loss(lgk, p_ref, spec)
        ste = gcn.init_state(E[idx], [W[k:k + 1] for W in Ws])
        gcn.train(lgk, ste, spec_exact, wl.epochs)
        tot_exact, _ = gcn.loss(lgk, gcn.forward(lgk, ste.E, ste.Ws, spec_exact)["p"], spec_exact)
        sensitivity = abs(tot_ref - tot_exact) / abs(tot_ref)
        p32 = p_ref.astype(np.float32)
        x_ref = cb.repair(sub.n, sub.rowptr, sub.col, None, p32, cb.round_probs(p32), "local")
        feas_ref = cb.count_conflicts(sub.n, sub.rowptr, sub.col, None, x_ref, "local") == 0
        feas_dev = cb.count_conflicts(sub.n, sub.rowptr, sub.col, None, x_dev[idx], "local") == 0
        size_ref, size_dev = int(x_ref.sum()), int(x_dev[idx].sum())
        print(f"c4 subgraph {k} ({sub.n} nodes) after {wl.epochs} epochs: loss {tot_ref:.2f} (without roundings "
              f"{tot_exact:.2f}: {sensitivity:.1e}) device {per_dev[k]:.2f}; set size {size_ref} device {size_dev}; "
              f"p rel {rel(p_dev[idx], p_ref):.2e} l2 {rel_l2(p_dev[idx], p_ref):.2e}", flush=True)
        bound = 1e-2 if sensitivity < 1e-3 else 5e-2
        assert abs(per_dev[k] - tot_ref) <= bound * abs(tot_ref)
        assert feas_ref and feas_dev
        assert abs(size_dev - size_ref) <= max(1, bound * size_ref)
        sum_ref += tot_ref
        sum_dev += per_dev[k]
    print(f"c4 sampled subgraphs together: loss {sum_ref:.2f} device {sum_dev:.2f}", flush=True)
    assert abs(sum_dev - sum_ref) <= 1e-2 * abs(sum_ref)
    ctx.destroy()


@pytest.mark.timeout(600)
def test_c4_as_one_subgraph_scaled(gco):
    """The stress variant with nothing cut (one subgraph holds the whole graph: more and
    longer pre-reduced rows, one weight set fed by hundreds of workgroup partials), at a
    tenth of c4's size so that the checker's full comparison stays short."""
    wl = inputs.make_workload("c4p1", scale=0.1)
    print("c4p1/10", inputs.describe(wl), flush=True)
    ctx, spec, lg, E, Ws = setup(gco, wl)
    fixed_weight_checks(ctx, spec, lg, E, Ws, "c4p1/10")
    got = ctx.train(5)
    st = gcn.init_state(E, Ws)
    want, _ = gcn.train(lg, st, spec, 5)
    assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
    ctx.set_params(E, Ws)
    np.testing.assert_array_equal(ctx.train(5), got)
    check_readout(ctx, wl, "local")
    ctx.destroy()


def subgraph_alone(wl, k):
    """Subgraph k of a workload as a graph of its own (nodes renumbered in ascending id)."""
    g = wl.graph
    row = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    idx = np.flatnonzero(wl.part == k)
    pos = -np.ones(g.n, dtype=np.int64)
    pos[idx] = np.arange(idx.shape[0])
    keep = (wl.part[row] == k) & (wl.part[g.col] == k)
    sub = inputs.from_edges(idx.shape[0], pos[row[keep]], pos[g.col[keep]])
    return idx, sub


C5_SAMPLE = (0, 77, 130, 255)


@pytest.mark.timeout(1200)
def test_c5_regular_graph_sampled_subgraphs(gco):
    """2 M nodes, 50-regular, 256 subgraphs, width 128.  The checker runs four sampled
    subgraphs one by one (subgraphs are independent: Sec. 3.3); the device trains all 256
    at once.  Fixed-weight comparison, then a ten-epoch trajectory of each sampled
    subgraph's own loss."""
    wl = inputs.make_workload("c5")
    print("c5", inputs.describe(wl), flush=True)
    g = wl.graph
    E, Ws = inputs.init_params(g.n, wl.part, wl.num_parts, wl.num_layers, wl.dim, wl.seed)
    ctx = gco.Context(problem=wl.problem, num_layers=wl.num_layers, dim=wl.dim,
                      storage=wl.storage, lr=wl.lr)
    ctx.upload_graph(g.n, g.rowptr, g.col, wl.part, wl.num_parts)
    ctx.set_params(E, Ws)
    ctx.forward()
    p = ctx.get_probs()
    _, per = ctx.loss()
    H = [None] + [ctx.get_hidden(l) for l in range(1, wl.num_layers)]
    dE, dWs = ctx.get_grads()
    spec = gcn.Spec(problem=wl.problem, num_layers=wl.num_layers, lr=wl.lr, storage="bf16")
    alone = {}
    for k in C5_SAMPLE:
        idx, sub = subgraph_alone(wl, k)
        lgk = gcn.local_graph(sub.n, sub.rowptr, sub.col, None, 1, "sym")
        Ek, Wk = E[idx], [W[k:k + 1] for W in Ws]
        alone[k] = (idx, lgk, Ek, Wk)
        label = f"c5[{k}]"
        want = parity.checker_side(lgk, Ek, Wk, spec)
        cache = want["cache"]
        assert rel(p[idx], cache["p"]) <= 2e-2
        tot, _ = gcn.loss(lgk, cache["p"], spec)
        assert abs(per[k] - tot) <= 2e-2 * abs(tot)
        for l in range(1, wl.num_layers):
            parity.compare_hidden(want, H[l][idx], l, label=label)
        parity.compare_gradient("dL/dE", dE[idx], want["gE"], want["sE"], label=label)
        for l in range(wl.num_layers):
            parity.compare_gradient(f"dL/dW_{l + 1}", dWs[l][k], want["gWs"][l][0], want["sWs"][l][0], label=label)
        print(f"c5 subgraph {k}: {idx.shape[0]} nodes ok", flush=True)
    u, v = ctx.cut_edges()
    wu, wv = cb.cut_edges_vectorised(g.n, g.rowptr, g.col, wl.part)
    np.testing.assert_array_equal(u, wu)
    np.testing.assert_array_equal(v, wv)
    del u, v, wu, wv
    # the configured 50 epochs of all 256 subgraphs, one at a time (the per-subgraph loss
    # belongs to the parameters before the step); the checker trains each sampled subgraph
    # alone.  Trajectory within 2e-2 throughout; at the end the loss within 1 %.
    got = []
    for e in range(wl.epochs):
        got.append(ctx.loss()[1][list(C5_SAMPLE)])
        ctx.train(1, return_loss=False)
    got = np.array(got)
    _, per_end = ctx.loss()
    x, obj, _, _ = ctx.round_repair(0.5, "local")
    assert obj == cb.cut_value(g.n, g.rowptr, g.col, wl.part, x, "all")
    for q, k in enumerate(C5_SAMPLE):
        idx, lgk, Ek, Wk = alone[k]
        _, sub = subgraph_alone(wl, k)
        st = gcn.init_state(Ek, Wk)
        want, _ = gcn.train(lgk, st, spec, wl.epochs)
        p_ref = gcn.forward(lgk, st.E, st.Ws, spec)["p"]
        end_ref, _ = gcn.loss(lgk, p_ref, spec)
        cut_ref = cb.cut_value(sub.n, sub.rowptr, sub.col, None, cb.round_probs(p_ref.astype(np.float32)), "all")
        cut_dev = cb.cut_value(sub.n, sub.rowptr, sub.col, None, x[idx], "all")
        print(f"c5 subgraph {k}: loss {want[0]:.2f} -> {end_ref:.2f} (device {got[0, q]:.2f} -> {per_end[k]:.2f}), "
              f"worst rel over the trajectory {np.abs(got[:, q] - want).max() / np.abs(want).max():.2e}; "
              f"cut {cut_ref} device {cut_dev}", flush=True)
        assert np.abs(got[:, q] - want).max() <= 2e-2 * np.abs(want).max()
        assert abs(per_end[k] - end_ref) <= 1e-2 * abs(end_ref)
        # (the cut values are printed only: at this workload's initialisation and learning
        # rate 50 epochs leave every p within about 1e-2 of 0.5, so which side of 0.5 a
        # node falls on is decided by rounding noise on both sides)
    x, obj, _, _ = ctx.round_repair(0.5, "local")
    assert obj == cb.cut_value(g.n, g.rowptr, g.col, wl.part, x, "all")
    ctx.destroy()


@pytest.mark.timeout(600)
def test_louvain_partition_end_to_end(gco):
    """Sec. 3.1 feeding Sec. 3.2: the library's modularity partitioner on the c3-shaped graph
    (ids equal to the checker's one by one), its communities packed into 16 subgraphs, that
    partition uploaded, and the training step compared with the checker at fixed weights
    and over ten epochs.  Packing never cuts an edge, so the cross edges are exactly the
    edges between different communities."""
    from oracle import louvain as lv
    wl = inputs.make_workload("c3")
    g = wl.graph
    comm, C, q = gco.louvain(g.n, g.rowptr, g.col)
    want, wantC = lv.louvain(g.n, g.rowptr, g.col)
    np.testing.assert_array_equal(comm, want)
    assert C == wantC
    want = np.asarray(want)
    assert abs(q - lv.modularity(g.n, g.rowptr, g.col, want)) <= 1e-12
    part, P = gco.pack_parts(comm, C, 16)
    want_part, wantP = lv.pack_parts(list(want), wantC, 16)
    np.testing.assert_array_equal(part, want_part)
    assert P == wantP and P <= 16
    E, Ws = inputs.init_params(g.n, part, P, wl.num_layers, wl.dim, wl.seed)
    Ws = [W * 1.5 for W in Ws]
    E = (E * 5).astype(np.float32)
    ctx = gco.Context(problem="mis", num_layers=wl.num_layers, dim=wl.dim, storage="bf16", lr=wl.lr)
    ctx.upload_graph(g.n, g.rowptr, g.col, part, P)
    ctx.set_params(E, Ws)
    info = ctx.graph_info()
    e = g.edges()
    assert info["m_cut"] == int((comm[e[:, 0]] != comm[e[:, 1]]).sum())
    bfs = int((wl.part[e[:, 0]] != wl.part[e[:, 1]]).sum())
    print(f"louvain: {C} communities, Q = {q:.4f}; cross edges {info['m_cut']} of {g.m} "
          f"(BFS region growing: {bfs})", flush=True)
    assert info["m_cut"] < bfs
    spec = gcn.Spec(problem="mis", num_layers=wl.num_layers, lr=wl.lr, storage="bf16")
    lg = gcn.local_graph(g.n, g.rowptr, g.col, part, P, "sym")
    parity.compare_bf16_run(ctx, lg, E, Ws, spec, label="c3/louvain")
    got = ctx.train(10)
    st = gcn.init_state(E, Ws)
    want_loss, _ = gcn.train(lg, st, spec, 10)
    assert np.abs(got - want_loss).max() <= 2e-2 * np.abs(want_loss).max()
    u, v = ctx.cut_edges()
    wu, wv = cb.cut_edges_vectorised(g.n, g.rowptr, g.col, part)
    np.testing.assert_array_equal(u, wu)
    np.testing.assert_array_equal(v, wv)
    ctx.destroy()
