"""GPU parity on the configured workloads, at their full sizes and in the launch
configuration the benchmark times.

  c1, c2 (fp32)  ten-epoch loss trajectory within 1e-4; after the configured number
                 of epochs the objective is within 1 % of the checker's and the
                 repaired solution is feasible on both sides
  c3, c4 (bf16)  probabilities, hidden activations and gradients at the initial
                 weights within 2e-2 (see test_gpu_parity for the ReLU-decision
                 rule); ten-epoch loss trajectory within 2e-2; integer read-out
                 bit-exact on the device's own probabilities
  c5 (bf16)      the same at fixed weights on a seeded sample of subgraphs, each
                 run through the checker alone (subgraphs are independent)
"""
import dataclasses

import numpy as np
import pytest

from oracle import combinatorial as cb
from oracle import gcn
from paper_2511_09261_amd import inputs

pytestmark = pytest.mark.gpu


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def setup(gco, wl):
    g = wl.graph
    E, Ws = inputs.init_params(g.n, wl.part, wl.num_parts, wl.num_layers, wl.dim, wl.seed)
    ctx = gco.Context(problem=wl.problem, num_layers=wl.num_layers, dim=wl.dim,
                      storage=wl.storage, lr=wl.lr)
    ctx.upload_graph(g.n, g.rowptr, g.col, wl.part, wl.num_parts)
    ctx.set_params(E, Ws)
    bf16 = wl.storage == "bf16"
    spec = gcn.Spec(problem=wl.problem, num_layers=wl.num_layers, lr=wl.lr,
                    storage="bf16" if bf16 else "exact", matrix_core_operands=bf16)
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


def fixed_weight_checks(ctx, spec, lg, E, Ws, tol=2e-2):
    L = spec.num_layers
    cache = gcn.forward(lg, E, Ws, spec)
    ctx.forward()
    p = ctx.get_probs()
    assert rel(p, cache["p"]) <= tol
    exact = gcn.forward(lg, E, Ws, dataclasses.replace(spec, storage="exact"))
    assert rel(p, exact["p"]) <= tol
    tot, per = ctx.loss()
    want_tot, want_per = gcn.loss(lg, cache["p"], spec)
    assert abs(tot - want_tot) <= tol * np.abs(want_per).sum()
    relu_on = [None]
    for l in range(1, L):
        H = ctx.get_hidden(l)
        assert rel(H, cache["H"][l]) <= tol
        relu_on.append(H > 0)
        assert ((H > 0) != (cache["H"][l] > 0)).mean() <= 1e-3
    gE, gWs = gcn.backward(lg, cache, Ws, spec, relu_on=relu_on)
    dE, dWs = ctx.get_grads()
    assert rel(dE, gE) <= tol
    for l in range(L):
        assert rel(dWs[l], gWs[l]) <= tol, f"layer {l + 1}"


def test_c3_bf16_workload(gco):
    wl = inputs.make_workload("c3")
    ctx, spec, lg, E, Ws = setup(gco, wl)
    fixed_weight_checks(ctx, spec, lg, E, Ws)
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


@pytest.mark.timeout(900)
def test_c4_youtube_shaped_full_size(gco):
    """The benchmark's workload (1.13 M nodes, 64 subgraphs, 3 layers, width 64, bf16)."""
    wl = inputs.make_workload("c4")
    print("c4", inputs.describe(wl), flush=True)
    ctx, spec, lg, E, Ws = setup(gco, wl)
    fixed_weight_checks(ctx, spec, lg, E, Ws)
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
    # deterministic: the same ten epochs again give the same bits
    ctx.set_params(E, Ws)
    np.testing.assert_array_equal(ctx.train(10), got)
    check_readout(ctx, wl, "local")
    ctx.destroy()


@pytest.mark.timeout(600)
def test_c4_as_one_subgraph_scaled(gco):
    """The stress variant with nothing cut (one subgraph holds the whole graph: more and
    longer pre-reduced rows, one weight set fed by hundreds of workgroup partials), at a
    tenth of c4's size so that the checker's full comparison stays short."""
    wl = inputs.make_workload("c4p1", scale=0.1)
    print("c4p1/10", inputs.describe(wl), flush=True)
    ctx, spec, lg, E, Ws = setup(gco, wl)
    fixed_weight_checks(ctx, spec, lg, E, Ws)
    got = ctx.train(5)
    st = gcn.init_state(E, Ws)
    want, _ = gcn.train(lg, st, spec, 5)
    assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
    ctx.set_params(E, Ws)
    np.testing.assert_array_equal(ctx.train(5), got)
    check_readout(ctx, wl, "local")
    ctx.destroy()


@pytest.mark.timeout(900)
def test_c5_regular_graph_sampled_subgraphs(gco):
    """2 M nodes, 50-regular, 256 subgraphs, width 128.  The checker runs four
    sampled subgraphs one by one; the device trains all 256 at once."""
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
    spec = gcn.Spec(problem=wl.problem, num_layers=wl.num_layers, lr=wl.lr, storage="bf16",
                    matrix_core_operands=True)
    row = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    for k in (0, 77, 130, 255):
        idx = np.flatnonzero(wl.part == k)
        pos = -np.ones(g.n, dtype=np.int64)
        pos[idx] = np.arange(idx.shape[0])
        keep = (wl.part[row] == k) & (wl.part[g.col] == k)
        sub = inputs.from_edges(idx.shape[0], pos[row[keep]], pos[g.col[keep]])
        lgk = gcn.local_graph(sub.n, sub.rowptr, sub.col, None, 1, "sym")
        Ek, Wk = E[idx], [W[k:k + 1] for W in Ws]
        cache = gcn.forward(lgk, Ek, Wk, spec)
        assert rel(p[idx], cache["p"]) <= 2e-2
        tot, _ = gcn.loss(lgk, cache["p"], spec)
        assert abs(per[k] - tot) <= 2e-2 * abs(tot)
        relu_on = [None]
        for l in range(1, wl.num_layers):
            assert rel(H[l][idx], cache["H"][l]) <= 2e-2
            relu_on.append(H[l][idx] > 0)
        gE, gWs = gcn.backward(lgk, cache, Wk, spec, relu_on=relu_on)
        assert rel(dE[idx], gE) <= 2e-2
        for l in range(wl.num_layers):
            assert rel(dWs[l][k], gWs[l][0]) <= 2e-2
        print(f"c5 subgraph {k}: {idx.shape[0]} nodes ok", flush=True)
    u, v = ctx.cut_edges()
    wu, wv = cb.cut_edges_vectorised(g.n, g.rowptr, g.col, wl.part)
    np.testing.assert_array_equal(u, wu)
    np.testing.assert_array_equal(v, wv)
    ctx.train(2, return_loss=False)
    x, obj, _, _ = ctx.round_repair(0.5, "local")
    assert obj == cb.cut_value(g.n, g.rowptr, g.col, wl.part, x, "all")
    ctx.destroy()
