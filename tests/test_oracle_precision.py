"""Pins for the checker's reduced-precision pieces (CPU only): the bf16-storage
backward pass, the bound on how far a bf16 run may lie from the checker
(oracle/precision.py: forward_bounds) and the bound on what undecidable ReLU units can do
to a gradient (flip_slack).

Each is fixed to something other than itself:
  * forward_bounds against an emulation written here from the arithmetic model alone
    (torch's bfloat16 cast, numpy float32 running sums in shuffled orders);
  * flip_slack against pairs of weight settings that put chosen units at +eps and -eps:
    whatever the exact gradients of the two settings differ by is what a flip does;
  * the bf16-storage backward pass against central differences of the unrounded loss, on
    inputs whose pre-activations all stay clear of zero.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import gcn
from oracle import precision as pr
from tests import helpers as hp


def make(n, edges, part=None, P=1, norm="sym"):
    rowptr, col = hp.csr_from_edges(n, edges)
    return gcn.local_graph(n, rowptr, col, part, P, norm)


def bf16(x):
    """Round-to-nearest-even to bfloat16 by torch's cast (not the checker's routine)."""
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def graph_with_a_hub(n, rs, hub_deg):
    edges = hp.random_graph(n, 0.08, rs)
    edges += [(0, int(j)) for j in rs.choice(np.arange(1, n), hub_deg, replace=False)]
    return edges


def emulated_run(lg, E, Ws, L, rs):
    """One run in the stated arithmetic: bf16 storage and operands, A_hat entries as two
    bf16 pieces, every sum a float32 running sum in a shuffled order."""
    n, d = E.shape
    A = lg.A_hat.tocsr()
    part = lg.part
    H = bf16(E)
    Zs, Hs = [None], [H]
    for l in range(1, L):
        Wb = bf16(Ws[l - 1])
        agg = np.zeros((n, d), dtype=np.float32)
        for i in range(n):
            cols = A.indices[A.indptr[i]:A.indptr[i + 1]]
            vals = A.data[A.indptr[i]:A.indptr[i + 1]].astype(np.float32)
            hi = bf16(vals)
            lo = bf16(vals - hi)
            terms = [(c, v) for c, v in zip(cols, hi)] + [(c, v) for c, v in zip(cols, lo)]
            rs.shuffle(terms)
            acc = np.zeros(d, dtype=np.float32)
            for c, v in terms:
                acc = (acc + np.float32(v) * H[c]).astype(np.float32)
            agg[i] = acc
        aggb = bf16(agg)
        Z = np.zeros((n, d), dtype=np.float32)
        for i in range(n):
            order = rs.permutation(d)
            acc = np.zeros(d, dtype=np.float32)
            for f in order:
                acc = (acc + aggb[i, f] * Wb[part[i], f, :]).astype(np.float32)
            Z[i] = acc
        H = bf16(np.maximum(Z, 0))
        Zs.append(Z)
        Hs.append(H)
    return Zs, Hs


@pytest.mark.parametrize("seed,norm", [(0, "sym"), (1, "mean"), (2, "sym")])
def test_forward_bounds_cover_an_emulated_bf16_run(seed, norm):
    rs = np.random.RandomState(seed)
    n, d, P, L = 70, 8, 2, 3
    edges = graph_with_a_hub(n, rs, 45)
    part = rs.randint(0, P, n)
    lg = make(n, edges, part, P, norm)
    E = rs.normal(0, 0.5, (n, d)).astype(np.float32)
    Ws = [rs.uniform(-0.8, 0.8, (P, d, d if l < L else 1)).astype(np.float32) for l in range(1, L + 1)]
    spec = gcn.Spec(num_layers=L, norm=norm, storage="bf16")
    cache = gcn.forward(lg, E, Ws, spec)
    b = pr.forward_bounds(lg, cache, Ws, spec)
    assert not b["dH"][0].any()                                  # the rounded embedding is common ground
    flips = 0
    for rep in range(4):
        Zs, Hs = emulated_run(lg, E, Ws, L, np.random.RandomState(100 * seed + rep))
        for l in range(1, L):
            assert (np.abs(Zs[l] - cache["Z"][l]) <= b["dZ"][l]).all()
            assert (np.abs(Hs[l] - cache["H"][l]) <= b["dH"][l]).all()
            differ = (Zs[l] > 0) != (cache["Z"][l] > 0)
            assert not (differ & ~b["amb"][l]).any()             # certain decisions are certain
            flips += int(differ.sum())
    # ... and the bounds are no wider than the model needs.  Layer 1: a unit in the last
    # place of fp32 times a small multiple of the number of terms.  Later layers inherit
    # stored values that may sit one bf16 step apart, so their bound is of the size of a
    # bf16 rounding step of the terms (2^-8), not more.
    for l in range(1, L):
        scale = np.abs(cache["Agg"][l]) @ np.ones((d, d)) * 0.8 + 1e-30
        assert np.median(b["dZ"][l] / scale) < (2e-4 if l == 1 else 2.0 ** -8)
        assert b["amb"][l].mean() < 0.02
    assert (b["dH"][1] == 0).mean() > 0.75                       # most stored values are certain


def test_forward_bounds_see_the_degree_and_earlier_layers():
    """A longer row sums more terms, so its aggregate is less certain and more often within
    reach of a bf16 rounding boundary; an uncertain stored value of layer 1 widens the
    bounds of the rows that gather it in layer 2."""
    rs = np.random.RandomState(5)
    stars, leaves, d, L = 40, 300, 4, 3
    n = stars * (leaves + 1)
    hubs = np.arange(stars) * (leaves + 1)
    edges = [(int(h), int(h) + j) for h in hubs for j in range(1, leaves + 1)]
    rowptr, col = hp.csr_from_edges(n, edges)
    lg = gcn.local_graph(n, rowptr, col, None, 1, "sym")
    E = rs.normal(0, 0.5, (n, d)).astype(np.float32)
    Ws = [rs.uniform(-0.8, 0.8, (1, d, d if l < L else 1)).astype(np.float32) for l in range(1, L + 1)]
    spec = gcn.Spec(num_layers=L, storage="bf16")
    cache = gcn.forward(lg, E, Ws, spec)
    b = pr.forward_bounds(lg, cache, Ws, spec)
    is_hub = np.zeros(n, dtype=bool)
    is_hub[hubs] = True
    # layer 1 (certain inputs): beyond the transform's own summation term, the bound holds
    # only what aggregates within reach of a rounding boundary add
    own = 4.0 * d * 2.0 ** -24 * (np.abs(cache["Agg"][1]) @ np.abs(gcn.round_bf16(Ws[0][0])))
    reached = (b["dZ"][1] > own * (1 + 1e-9)).any(axis=1)
    assert reached[is_hub].mean() > 0.5 and reached[~is_hub].mean() < 0.1
    # layer 2: rows that gather only certain values of H_1 and whose own aggregate is clear
    # of every boundary carry the summation term alone; rows that gather an uncertain value
    # carry more
    certain_in = (lg.A_hat @ b["dH"][1]).sum(axis=1) == 0
    own2 = 4.0 * d * 2.0 ** -24 * (np.abs(cache["Agg"][2]) @ np.abs(gcn.round_bf16(Ws[1][0])))
    wider = b["dZ"][2] > own2 * (1 + 1e-9)
    agg2 = lg.A_hat @ cache["H"][1]
    t_agg = (2.0 ** -18 + 2.0 ** -21 + 4.0 * (2.0 * lg.deg + 4.0) * 2.0 ** -24)[:, None]
    d2 = t_agg * (lg.A_hat @ np.abs(cache["H"][1]))
    stable = (gcn.round_bf16(agg2 + d2) == gcn.round_bf16(agg2 - d2)).all(axis=1)
    assert (certain_in & stable).sum() > 100 and not wider[certain_in & stable].any()
    assert (~certain_in).sum() > 100 and wider[~certain_in].any(axis=1).mean() > 0.5
    # a smaller safety factor gives bounds that are nowhere larger and somewhere smaller
    b1 = pr.forward_bounds(lg, cache, Ws, spec, safety=1.0)
    for l in (1, 2):
        assert (b1["dZ"][l] <= b["dZ"][l]).all() and (b1["dZ"][l] < b["dZ"][l]).any()


def small_integer_network(n, d, L, P, rs, norm):
    """Inputs on which every sum of the forward pass is exact in fp32: a graph whose
    normalised entries are powers of two (every node has 3 neighbours inside its subgraph:
    1/4 everywhere), embeddings in {-2..2}, weights in {-1, 0, 1}."""
    per = n // P
    edges = []
    for k in range(P):                                   # a 3-regular circulant per subgraph
        base = k * per
        for i in range(per):
            edges.append((base + i, base + (i + 1) % per))
            if i < per // 2:
                edges.append((base + i, base + i + per // 2))
    part = np.repeat(np.arange(P), per)
    rowptr, col = hp.csr_from_edges(n, edges)
    lg = gcn.local_graph(n, rowptr, col, part, P, norm)
    E = rs.randint(-2, 3, (n, d)).astype(np.float32)
    Ws = [rs.randint(-1, 2, (P, d, d if l < L else 1)).astype(np.float32) for l in range(1, L + 1)]
    return lg, E, Ws


@pytest.mark.parametrize("norm", ["sym", "mean"])
def test_forward_bounds_vanish_where_fp32_sums_are_exact(norm):
    """On a small-integer network no sum can round, whatever its order: the bounds are zero
    everywhere, no unit is undecidable (pre-activations that are exactly zero included), and
    the emulated runs reproduce the checker's activations bit for bit.  One embedding entry
    that is not on the grid brings the error terms back for the rows that gather it."""
    rs = np.random.RandomState(4)
    n, d, L, P = 96, 8, 3, 2
    lg, E, Ws = small_integer_network(n, d, L, P, rs, norm)
    assert set(np.unique(lg.A_hat.data)) == {0.25}
    spec = gcn.Spec(num_layers=L, norm=norm, storage="bf16")
    cache = gcn.forward(lg, E, Ws, spec)
    b = pr.forward_bounds(lg, cache, Ws, spec)
    for l in range(1, L):
        assert not b["dZ"][l].any() and not b["dH"][l].any() and not b["amb"][l].any()
        assert (cache["Z"][l] == 0).any()                # exact zeros occur and are settled
    for rep in range(3):
        Zs, Hs = emulated_run(lg, E, Ws, L, np.random.RandomState(rep))
        for l in range(1, L):
            np.testing.assert_array_equal(Zs[l], cache["Z"][l])
            np.testing.assert_array_equal(Hs[l], cache["H"][l])
    E2 = E.copy()
    E2[5, 3] = 1.0 + 2.0 ** -7 + 1e-3                    # rounds to a bf16 value with a low last bit
    cache2 = gcn.forward(lg, E2, Ws, spec)
    b2 = pr.forward_bounds(lg, cache2, Ws, spec)
    # still exact: the rounded value is on a finer grid, and the sums stay far below 2^24 units of it
    assert not b2["dZ"][1].any()
    E2[5, 3] = 1e-12                                      # a grid 2^-47 fine: the sums overflow 24 bits of it
    cache2 = gcn.forward(lg, E2, Ws, spec)
    b2 = pr.forward_bounds(lg, cache2, Ws, spec)
    assert b2["dZ"][1].any()


def test_lowest_bit_exponent():
    got = pr._lowest_bit_exponent(np.array([4.0, 12.0, 0.75, -0.25, 3.0, 1.0 + 2.0 ** -40, 0.0]))
    np.testing.assert_array_equal(got, [2, 2, -2, -2, 0, -40, pr._NO_BIT])


def test_row_grid_of_aggregate_is_the_minimum_over_the_row():
    import scipy.sparse as sp
    A = sp.csr_matrix(np.array([[0.5, 0.25, 0.0], [0.0, 1.0, 0.125], [0.0, 0.0, 0.0]]))
    H = np.array([[4.0, 0.0], [3.0, 0.5], [0.0, 0.0]])
    # row 0: 0.5 * {4, 0} -> 2^1 ; 0.25 * {3, 0.5} -> 2^-3          => -3
    # row 1: 1 * {3, 0.5} -> 2^-1 ; 0.125 * zero row -> no bit       => -1
    # row 2: no entries                                               => none
    np.testing.assert_array_equal(pr._row_grid_of_aggregate(A, H), [-3, -1, pr._NO_BIT])


def _put_unit_at(lg, cache_fn, Ws, l, i, o, f, value):
    """Weights equal to Ws except W_l[k(i), f, o], moved so that Z_l[i, o] == value."""
    W2 = [W.copy() for W in Ws]
    cache = cache_fn(W2)
    k = lg.part[i]
    W2[l - 1][k, f, o] += (value - cache["Z"][l][i, o]) / cache["Agg"][l][i, f]
    return W2


@pytest.mark.parametrize("L,layer", [(2, 1), (3, 2), (3, 1)])
@pytest.mark.parametrize("norm", ["sym", "mean"])
def test_flip_slack_covers_what_flipped_units_do(L, layer, norm):
    """Three units of one layer (in two subgraphs) are put at +eps or -eps by moving one
    weight each; the exact gradients of the 8 settings differ only through those three
    decisions (up to O(eps)).  Every pairwise difference must lie under the slack computed
    from one of them with exactly those units flagged."""
    rs = np.random.RandomState(10 * L + layer)
    n, d, P = 24, 4, 3
    edges = hp.random_graph(n, 0.2, rs)
    part = np.arange(n) % P
    lg = make(n, edges, part, P, norm)
    spec = gcn.Spec(problem="mis", num_layers=L, norm=norm)
    E = rs.normal(0, 0.5, (n, d))
    Ws = [rs.uniform(-0.8, 0.8, (P, d, d if l < L else 1)) for l in range(1, L + 1)]
    units = [(3, 0), (6, 1), (10, 2)]            # (row, column): subgraphs 0, 0, 1; distinct columns
    eps = 1e-9
    grads = []
    for signs in itertools.product([1.0, -1.0], repeat=3):
        W2 = Ws
        for (i, o), sgn in zip(units, signs):
            W2 = _put_unit_at(lg, lambda W: gcn.forward(lg, E, W, spec), W2, layer, i, o, f=o, value=sgn * eps)
        cache = gcn.forward(lg, E, W2, spec)
        for (i, o), sgn in zip(units, signs):
            assert abs(cache["Z"][layer][i, o] - sgn * eps) < 1e-12
        trace = {}
        gE, gWs = gcn.backward(lg, cache, W2, spec, trace=trace)
        grads.append((cache, trace["G_H"], W2, gE, gWs))
    amb = [None] + [np.zeros((n, d), dtype=bool) for _ in range(1, L)]
    for i, o in units:
        amb[layer][i, o] = True
    cache, G_H, W2, gE0, gW0 = grads[0]
    sE, sWs = pr.flip_slack(lg, cache, G_H, W2, spec, amb)
    smooth = 1e-7                                    # the settings themselves differ by O(eps)
    worst_E, worst_W = 0.0, 0.0
    for (_, _, _, gEa, gWa), (_, _, _, gEb, gWb) in itertools.combinations(grads, 2):
        assert (np.abs(gEa - gEb) <= sE + smooth).all()
        worst_E = max(worst_E, np.abs(gEa - gEb).max())
        for l in range(L):
            assert (np.abs(gWa[l] - gWb[l]) <= sWs[l] + smooth).all()
        worst_W = max(worst_W, np.abs(gWa[layer - 1] - gWb[layer - 1]).max())
    # the bound is attained by the weight gradient of the flipped layer, and it is not idle
    assert worst_W > 1e-4 and abs(worst_W - sWs[layer - 1].max()) <= 1e-6
    assert worst_E > 1e-5 and sE.max() <= 50 * worst_E
    # nothing leaks to what the units cannot reach: subgraph 2, the scalar layer, later layers
    assert not sE[part == 2].any()
    assert not sWs[L - 1].any()
    for l in range(L - 1):
        assert not sWs[l][2].any()
        if l + 1 > layer:
            assert not sWs[l].any()
    # without flagged units there is no slack at all
    none = [None] + [np.zeros((n, d), dtype=bool) for _ in range(1, L)]
    sE, sWs = pr.flip_slack(lg, cache, G_H, W2, spec, none)
    assert not sE.any() and not any(s.any() for s in sWs)


def test_flip_slack_with_shared_weights_and_a_subset():
    rs = np.random.RandomState(3)
    n, d, P, L = 20, 3, 2, 3
    edges = hp.random_graph(n, 0.25, rs)
    part = np.arange(n) % P
    lg = make(n, edges, part, P)
    spec = gcn.Spec(num_layers=L, weight_sharing=True)
    E = rs.normal(0, 0.5, (n, d))
    Ws = [rs.uniform(-0.8, 0.8, (1, d, d if l < L else 1)) for l in range(1, L + 1)]
    cache = gcn.forward(lg, E, Ws, spec)
    trace = {}
    gcn.backward(lg, cache, Ws, spec, trace=trace)
    amb = [None] + [np.zeros((n, d), dtype=bool) for _ in range(1, L)]
    amb[2][4, 1] = True                              # node 4 is in subgraph 0
    sE, sWs = pr.flip_slack(lg, cache, trace["G_H"], Ws, spec, amb)
    assert sWs[1][0].any() and sWs[0][0].any() and not sE[part == 1].any()
    only1 = np.array([False, True])
    _, sW1 = pr.flip_slack(lg, cache, trace["G_H"], Ws, spec, amb, active=only1)
    assert not any(s.any() for s in sW1)             # subgraph 0 does not feed the shared gradient then


def _clear_of_zero(lg, E, Ws, spec, margin):
    cache = gcn.forward(lg, E, Ws, spec)
    for l in range(1, spec.num_layers):
        S = np.zeros_like(cache["Z"][l])
        for k, idx in enumerate(lg.members):
            S[idx] = np.abs(cache["Agg"][l][idx]) @ np.abs(Ws[l - 1][0 if spec.weight_sharing else k])
        if (np.abs(cache["Z"][l]) <= margin * S).any():
            return False
    return True


@pytest.mark.parametrize("problem,norm,L,P,share", [
    ("mis", "sym", 3, 2, False), ("maxcut", "mean", 3, 1, False), ("mis", "mean", 2, 3, True),
    ("maxcut", "sym", 2, 2, False)])
def test_bf16_backward_against_central_differences_of_the_unrounded_loss(problem, norm, L, P, share):
    """Rounding moves every stored value by at most 2^-9 of itself, so where no
    pre-activation comes near zero the bf16-storage gradient must be the derivative of
    the unrounded loss to within a few such steps (4e-2 of the tensor's largest entry: these
    tiny sums cancel more than the workloads' do): E and every W_l, entry by entry."""
    n, d = 14, 3
    for seed in range(2000):
        rs = np.random.RandomState(seed)
        edges = hp.random_graph(n, 0.25, rs)
        part = rs.randint(0, P, n)
        lg = make(n, edges, part, P, norm)
        E = rs.normal(0, 0.5, (n, d))
        Ws = [rs.uniform(-0.8, 0.8, (1 if share else P, d, d if l < L else 1)) for l in range(1, L + 1)]
        exact = gcn.Spec(problem=problem, num_layers=L, norm=norm, weight_sharing=share)
        if _clear_of_zero(lg, E, Ws, exact, margin=0.03):
            break
    else:
        raise AssertionError("no input clear of zero found")
    spec = gcn.Spec(problem=problem, num_layers=L, norm=norm, weight_sharing=share, storage="bf16")
    cache = gcn.forward(lg, E, Ws, spec)
    ref = gcn.forward(lg, E, Ws, exact)
    for l in range(1, L):                               # same decisions in both modes
        np.testing.assert_array_equal(cache["Z"][l] > 0, ref["Z"][l] > 0)
    # no unit is ambiguous under the run-to-run bound either
    b = pr.forward_bounds(lg, cache, Ws, spec)
    assert not any(a.any() for a in b["amb"][1:])
    gE, gWs = gcn.backward(lg, cache, Ws, spec)
    h = 1e-6

    def total(E_, Ws_):
        return gcn.loss(lg, gcn.forward(lg, E_, Ws_, exact)["p"], exact)[0]

    def fd(arr, f):
        g = np.zeros_like(arr)
        for ix in np.ndindex(arr.shape):
            a = arr.copy(); a[ix] += h
            c = arr.copy(); c[ix] -= h
            g[ix] = (f(a) - f(c)) / (2 * h)
        return g

    fE = fd(E, lambda a: total(a, Ws))
    assert np.abs(fE - gE).max() <= 4e-2 * np.abs(fE).max()
    assert np.abs(fE - gE).max() > 0                    # the mode does round something
    for l in range(L):
        def with_w(a, l=l):
            W2 = list(Ws); W2[l] = a
            return total(E, W2)
        fW = fd(Ws[l], with_w)
        assert np.abs(fW - gWs[l]).max() <= 4e-2 * np.abs(fW).max(), l


def test_bf16_backward_rounds_the_gradient_kept_between_hidden_layers():
    """L = 3: dL/dZ_1 is stored between the two hidden layers, so the embedding gradient
    is A_hat^T (bf16(G_Z1) W_1^T): rebuilt here from the trace with torch's cast."""
    rs = np.random.RandomState(2)
    n, d, L = 16, 4, 3
    lg = make(n, hp.random_graph(n, 0.25, rs))
    E = rs.normal(0, 0.5, (n, d))
    Ws = [rs.uniform(-0.8, 0.8, (1, d, d if l < L else 1)) for l in range(1, L + 1)]
    spec = gcn.Spec(num_layers=L, storage="bf16")
    cache = gcn.forward(lg, E, Ws, spec)
    trace = {}
    gE, gWs = gcn.backward(lg, cache, Ws, spec, trace=trace)
    G_Z1 = bf16(trace["G_H"][1] * (cache["Z"][1] > 0)).astype(np.float64)
    np.testing.assert_allclose(gE, lg.A_hat.T @ (G_Z1 @ Ws[0][0].T), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(gWs[0][0], cache["Agg"][1].T @ G_Z1, rtol=1e-12, atol=1e-300)
    # the last hidden layer's gradient is consumed unrounded
    G_Z2 = trace["G_H"][2] * (cache["Z"][2] > 0)
    np.testing.assert_allclose(gWs[1][0], cache["Agg"][2].T @ G_Z2, rtol=1e-12, atol=1e-300)
    # and both dense-transform operands of the forward pass are bf16 values
    for l in (1, 2):
        np.testing.assert_array_equal(bf16(cache["Agg"][l]).astype(np.float64), cache["Agg"][l])
    np.testing.assert_array_equal(cache["Z"][1], cache["Agg"][1] @ bf16(Ws[0][0]).astype(np.float64))
