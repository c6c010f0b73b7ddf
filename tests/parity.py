"""What the GPU parity tests share: the norms in which tensors are compared and the
comparison of a bf16-storage run with the checker.

The bf16 comparison never hands a device value to the checker.  The checker computes, from
its own forward pass, which ReLU decisions are certain and how far the undecidable ones can
move each gradient entry (oracle/precision.py); the device must take every certain
decision as the checker does, and each gradient entry must match within
    tol * max|gradient tensor|  +  that entry's slack,
where the slack is zero for every entry no undecidable unit reaches.
"""
import numpy as np

from oracle import gcn
from oracle import precision as pr

TOL_BF16 = 2e-2
# share of hidden units whose ReLU decision the arithmetic model cannot settle: a property
# of the inputs alone (computed by the checker), asserted so that the comparison cannot
# silently turn vacuous.  First hidden layer: a few in ten thousand to a few in a thousand;
# later layers gather stored values that may already sit one bf16 step apart: several in a
# hundred, and a fifth where thousands of rows gather the row of one long-row hub.
MAX_AMBIGUOUS_SHARE = (None, 1e-2, 0.5)


def rel(a, b):
    """max |a - b| / max |b|"""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def rel_l2(a, b):
    """||a - b||_2 / ||b||_2"""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def checker_side(lg, E, Ws, spec, extra=None, active=None):
    """Everything the checker contributes to a bf16 comparison, from the inputs alone."""
    assert spec.storage == "bf16"
    cache = gcn.forward(lg, E, Ws, spec)
    bounds = pr.forward_bounds(lg, cache, Ws, spec)
    trace = {}
    gE, gWs = gcn.backward(lg, cache, Ws, spec, extra, active=active, trace=trace)
    sE, sWs = pr.flip_slack(lg, cache, trace["G_H"], Ws, spec, bounds["amb"], active=active)
    return {"cache": cache, "bounds": bounds, "gE": gE, "gWs": gWs, "sE": sE, "sWs": sWs}


def compare_hidden(want, H_dev, l, rows=None, tol=TOL_BF16, label=""):
    """Hidden activations of layer l: values within tol, every certain ReLU decision equal."""
    cache, b = want["cache"], want["bounds"]
    H_ref, Z, amb, dH = cache["H"][l], cache["Z"][l], b["amb"][l], b["dH"][l]
    if rows is not None:
        H_ref, Z, amb, dH = H_ref[rows], Z[rows], amb[rows], dH[rows]
    assert rel(H_dev, H_ref) <= tol, f"{label} H_{l}"
    differ = (H_dev > 0) != (Z > 0)
    wrong = differ & ~amb
    assert not wrong.any(), f"{label} layer {l}: {int(wrong.sum())} certain ReLU decisions differ"
    share = float(amb.mean())
    assert share <= MAX_AMBIGUOUS_SHARE[min(l, 2)], f"{label} layer {l}: {share:.2e} of the units are undecidable"
    outside = np.abs(H_dev - H_ref) > dH * (1 + 1e-6) + 1e-30
    print(f"{label} H_{l}: rel {rel(H_dev, H_ref):.2e} l2 {rel_l2(H_dev, H_ref):.2e}; undecidable "
          f"{int(amb.sum())} of {amb.size} ({share:.1e}), of which the device took {int(differ.sum())} "
          f"the other way; values outside the model's bound: {int(outside.sum())}", flush=True)
    return int(outside.sum())


def compare_gradient(name, got, ref, slack, tol=TOL_BF16, label="", plain=False):
    """plain: the entries must also match within the tolerance alone, slack or not (for inputs
    on which the undecidable units carry too little gradient to matter)."""
    got = np.asarray(got, dtype=np.float64)
    scale = np.abs(ref).max()
    excess = np.abs(got - ref) - slack
    loose = slack > tol * scale
    print(f"{label} {name}: rel {rel(got, ref):.2e} l2 {rel_l2(got, ref):.2e}; entries with slack "
          f"{int((slack > 0).sum())} of {slack.size}, with slack above the tolerance {int(loose.sum())}; "
          f"largest excess over the slack {excess.max() / max(scale, 1e-300):.2e} of max|g|", flush=True)
    assert excess.max() <= tol * scale, f"{label} {name}"
    if plain:
        assert rel(got, ref) <= tol, f"{label} {name} (without slack)"


def compare_bf16_run(ctx, lg, E, Ws, spec, extra=None, tol=TOL_BF16, label="", plain=False):
    """Forward probabilities, loss, hidden activations with their ReLU decisions, and all
    gradients of the device context ctx (parameters already set) against the checker."""
    import dataclasses
    L = spec.num_layers
    want = checker_side(lg, E, Ws, spec, extra)
    cache = want["cache"]
    ctx.forward()
    p = ctx.get_probs()
    exact = gcn.forward(lg, E, Ws, dataclasses.replace(spec, storage="exact"))
    print(f"{label} p: rel {rel(p, cache['p']):.2e} l2 {rel_l2(p, cache['p']):.2e}; against the unrounded "
          f"checker rel {rel(p, exact['p']):.2e}", flush=True)
    assert rel(p, cache["p"]) <= tol
    assert rel(p, exact["p"]) <= tol
    tot, per = ctx.loss()
    want_tot, want_per = gcn.loss(lg, cache["p"], spec, extra)
    assert abs(tot - want_tot) <= tol * max(1.0, np.abs(want_per).sum())
    assert abs(tot - gcn.loss(lg, exact["p"], spec, extra)[0]) <= tol * max(1.0, np.abs(want_per).sum())
    assert rel(per, want_per) <= tol * 10
    outside = 0
    for l in range(1, L):
        outside += compare_hidden(want, ctx.get_hidden(l), l, tol=tol, label=label)
    dE, dWs = ctx.get_grads()
    compare_gradient("dL/dE", dE, want["gE"], want["sE"], tol, label, plain)
    for l in range(L):
        compare_gradient(f"dL/dW_{l + 1}", dWs[l], want["gWs"][l], want["sWs"][l], tol, label, plain)
    assert outside == 0, f"{label}: {outside} stored activations lie outside the arithmetic model's bound"
    return want


def power_of_two_case(seed, d, L, hubs=(63, 255, 1023, 1023), ring_blocks=6, ring_size=500):
    """Inputs on which every sum of the forward pass is exact in fp32 in any order, so that a
    bf16-storage run must reproduce the checker bit for bit (oracle/precision.py certifies
    it: all bounds zero).  The normalised adjacency has only powers of two as entries under
    either normalisation when every |N(i)| + 1 is a power of four:
      * blocks of a 3-regular circulant graph (|N(i)| + 1 = 4);
      * wheels: a hub with 63, 255 or 1023 spokes whose other ends form a ring (hub: 64,
        256, 1024; rim nodes: 4), which also gives rows of every length class.
    Embeddings are integers in [-2, 2] (zero for the hubs, whose tiny entries would otherwise
    put a much finer grid under their neighbours' sums); weights are -1, 0, 1 times a power
    of two that keeps the activations of order one.  Subgraphs: the wheels share subgraph 0 and 1, the
    circulant blocks go round-robin over all P = 4.  Returns (graph, part, P, E, Ws)."""
    from paper_2511_09261_amd import inputs
    rs = np.random.RandomState(seed)
    us, vs, part = [], [], []
    n = 0
    P = 4
    hub_ids = []
    for q, m in enumerate(hubs):                         # wheel: hub n, rim n+1 .. n+m
        hub_ids.append(n)
        rim = n + 1 + np.arange(m)
        us += [np.full(m, n), rim]
        vs += [rim, n + 1 + (np.arange(m) + 1) % m]
        part += [q % 2] * (m + 1)
        n += m + 1
    for b in range(ring_blocks):
        size = ring_size + 2 * b                         # even sizes, not multiples of a tile
        i = np.arange(size)
        us += [n + i, n + i[: size // 2]]
        vs += [n + (i + 1) % size, n + i[: size // 2] + size // 2]
        part += [b % P] * size
        n += size
    g = inputs.from_edges(n, np.concatenate(us), np.concatenate(vs))
    part = np.asarray(part, dtype=np.int32)
    E = rs.randint(-2, 3, (n, d)).astype(np.float32)
    E[hub_ids] = 0
    scale = [2.0 ** -3] * (L - 1) + [2.0 ** -5]
    Ws = [(rs.randint(-1, 2, (P, d, d if l < L else 1)) * scale[l - 1]).astype(np.float32)
          for l in range(1, L + 1)]
    return g, part, P, E, Ws
