"""How far a reduced-precision run may lie from the checker, and what that can do
to a gradient (fp64, CPU, numpy).

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by tests, never by the
product path, no code shared with the HIP sources.

Why this exists.  The hidden layers of Eq. 3 end in a ReLU, so the backward pass of
Sec. 3.2 multiplies by the yes/no decision [Z > 0].  A run that accumulates in fp32, in
whatever order its kernels choose, reproduces the checker's Z only up to rounding; a unit
whose Z is zero to within that rounding may fall on either side, and one such unit moves a
whole gradient row by O(1).  The gradient of the loss is discontinuous there: neither side
is wrong.  Instead of asking the run under test which side it took, the checker

  1. bounds, by interval arithmetic over its own bf16-storage forward pass, how far a run
     in the stated arithmetic (below) can be from it: dZ_l >= |Z_l(run) - Z_l|,
     dH_l >= |H_l(run) - H_l| element by element       (forward_bounds);
  2. calls a unit ambiguous iff |Z_l| <= dZ_l: everywhere else the decision is certain and
     a run must agree with the checker;
  3. bounds, by propagating absolute values through the chain rule, how much any pattern
     of decisions on the ambiguous units can move each gradient entry   (flip_slack).

A gradient entry then has to match within the ordinary tolerance plus its own slack; the
slack is zero for every entry that no ambiguous unit reaches.

Arithmetic model of the run (bf16 storage, fp32 accumulate).  u = 2^-24.
  * H_0 = bf16(E): the same fp32 numbers rounded by the same rule on both sides, no error.
  * aggregate_i = sum_j A_hat_ij H_j over deg_i + 1 terms.  An entry of A_hat may be held
    as two bf16 pieces hi = bf16(a), lo = bf16(a - hi): |a - hi - lo| <= 2^-9 |a - hi| <=
    2^-18 |a|.  Scale factors are computed in fp32 (a few u: 2^-21 allowed).  Products of
    two bf16 numbers are exact in fp32.  The 2 (deg_i + 1) products are summed in fp32 in
    an unknown order (standard worst-case bound, n u times the sum of absolute values):
      |error| <= t_agg_i * (A_hat |H|)_i,   t_agg_i = 2^-18 + 2^-21 + c (2 deg_i + 4) u.
  * the aggregate is rounded to bf16 (operand of the dense transform); rounding is
    monotone, so bf16(x + e) lies between bf16(x - d) and bf16(x + d) for |e| <= d.
  * Z = aggregate_bf16 . W_bf16 over d terms, fp32 accumulation in any order:
      |error| <= t_w * (|aggregate| . |W|),   t_w = c d u.
  * H = bf16(max(Z, 0)), monotone again.
  * c = SAFETY = 4 leaves room for the order of additions inside a matrix instruction.
  * A sum whose terms are all multiples of 2^q and whose absolute values add up to less
    than 2^(24+q) is EXACT in fp32 in every order (each partial sum is such a multiple
    below 2^24 of them): it gets no error term.  Entries of A_hat that are bf16 numbers
    themselves (powers of two, say) have lo = 0 and no representation error.  On inputs
    built from small integers the whole forward pass is exact in this sense: a run must
    then reproduce the checker's stored activations bit for bit, and no decision is open
    (a pre-activation that is exactly zero is zero on both sides).
Uncertainty compounds: an aggregate that may round either way moves Z by a bf16 step of one
term, which may move a stored H, which the next layer gathers.  On generic inputs a few in
ten thousand units of a first hidden layer and one or two in a hundred of a second come out
undecidable; the slack they cause is what the comparison allows, no more.
"""
from __future__ import annotations

import numpy as np

from . import gcn

U32 = 2.0 ** -24
SAFETY = 4.0


def _abs_weights(lg, X, W, spec):
    """rows of subgraph k times |W[k]| (X is non-negative)."""
    out = np.zeros((lg.n, W.shape[2]))
    for k, idx in enumerate(lg.members):
        out[idx] = X[idx] @ np.abs(W[0] if spec.weight_sharing else W[k])
    return out


_NO_BIT = 4096      # exponent standing for "no set bit" (a zero entry): larger than any real one


def _lowest_bit_exponent(x):
    """Element-wise q such that x is an odd multiple of 2^q; _NO_BIT for zero entries.
    Entries are fp64 numbers."""
    x = np.asarray(x, dtype=np.float64)
    frac, exp = np.frexp(np.abs(x))                      # |x| = frac * 2^exp, frac in [0.5, 1)
    mant = (frac * 2.0 ** 53).astype(np.int64)           # 53-bit integer mantissa
    low = mant & -mant                                   # its lowest set bit
    tz = np.frexp(low.astype(np.float64))[1] - 1
    return np.where(x != 0, exp - 53 + tz, _NO_BIT).astype(np.int64)


def _row_grid_of_aggregate(A_hat, H):
    """Per row i of A_hat: q_i such that every product A_hat_ij H[j, f] is a multiple of
    2^q_i (the minimum over the row's entries of the entry's lowest bit plus the lowest bit
    found in the gathered row of H)."""
    row_bit = _lowest_bit_exponent(H).min(axis=1)
    term_bit = _lowest_bit_exponent(A_hat.data) + row_bit[A_hat.indices]
    # row-wise minimum of term_bit, as a row-wise maximum of a sparse matrix of 2^-term_bit
    M = A_hat.copy()
    M.data = np.exp2(-np.minimum(term_bit, 1000).astype(np.float64))     # 2^-1000 > 0 still
    top = np.asarray(M.max(axis=1).todense()).ravel()
    with np.errstate(divide="ignore"):
        return np.where(top > 0, -np.log2(top), _NO_BIT)


def forward_bounds(lg: gcn.LocalGraph, cache: dict, Ws, spec: gcn.Spec, safety: float = SAFETY) -> dict:
    """cache: gcn.forward(...) with spec.storage == "bf16".  Returns, per hidden layer l
    (lists indexed by l, entry 0 unused): dZ, dH as above and amb = (|Z| <= dZ, dZ > 0).
    safety is the constant c of the fp32 summation terms (see the module text)."""
    if spec.storage != "bf16":
        raise ValueError("bounds are defined for the bf16-storage forward pass")
    L = spec.num_layers
    d = cache["H"][0].shape[1]
    t_agg = (2.0 ** -18 + 2.0 ** -21 + safety * (2.0 * lg.deg + 4.0) * U32)[:, None]
    t_w = safety * d * U32
    entries_are_bf16 = bool((gcn.round_bf16(lg.A_hat.data) == lg.A_hat.data).all())
    dH = np.zeros_like(cache["H"][0])
    out = {"dZ": [None], "dH": [dH], "amb": [None]}
    for l in range(1, L):
        H_prev = cache["H"][l - 1]
        agg_exact = lg.A_hat @ H_prev
        abs_sum = lg.A_hat @ np.abs(H_prev)
        own = t_agg * abs_sum
        if entries_are_bf16:                             # sums that are exact in any order
            grid = _row_grid_of_aggregate(lg.A_hat, H_prev)[:, None]
            own[abs_sum < np.exp2(24.0 + np.minimum(grid, 900))] = 0.0
        d_agg = lg.A_hat @ dH + own
        d_aggb = gcn.round_bf16(agg_exact + d_agg) - gcn.round_bf16(agg_exact - d_agg)
        Wb = gcn.round_bf16(np.asarray(Ws[l - 1], dtype=np.float64))
        abs_sum = _abs_weights(lg, np.abs(cache["Agg"][l]), Wb, spec)
        own = t_w * abs_sum
        w_bit = _lowest_bit_exponent(Wb).min()
        grid = (_lowest_bit_exponent(cache["Agg"][l]).min(axis=1) + w_bit)[:, None]
        own[abs_sum < np.exp2(24.0 + np.minimum(grid, 900))] = 0.0
        dZ = _abs_weights(lg, d_aggb, Wb, spec) + own
        Z = cache["Z"][l]
        dH = gcn.round_bf16(np.maximum(Z + dZ, 0.0)) - gcn.round_bf16(np.maximum(Z - dZ, 0.0))
        out["dZ"].append(dZ)
        out["dH"].append(dH)
        out["amb"].append((np.abs(Z) <= dZ) & (dZ > 0))
    return out


def flip_slack(lg: gcn.LocalGraph, cache: dict, G_H: list, Ws, spec: gcn.Spec, amb: list, active=None):
    """Upper bound, entry by entry, on how far the gradients can move when the ReLU
    decisions of the units flagged in amb[l] are taken either way (all other decisions as
    the checker takes them).  G_H: the trace of gcn.backward.  Returns (sE, [sW_1..sW_L])
    shaped like the gradients.

    With D_l the bound on dL/dH_l (zero at the last hidden layer, whose incoming gradient
    does not pass a ReLU) and on_l = [Z_l > 0]:
      dG_Z = amb_l (|G_H_l| + D_l) + (1 - amb_l) on_l D_l
      sW_l = |Agg_l|^T dG_Z  (per subgraph),   D_{l-1} = A_hat^T (dG_Z |W_l|^T)."""
    on_k = np.ones(lg.num_parts, dtype=bool) if active is None else np.asarray(active, dtype=bool)
    L = spec.num_layers
    sWs = [np.zeros_like(np.asarray(W, dtype=np.float64)) for W in Ws]
    D = np.zeros_like(cache["H"][0])
    for l in range(L - 1, 0, -1):
        a = amb[l]
        on = cache["Z"][l] > 0.0
        dG_Z = np.where(a, np.abs(G_H[l]) + D, np.where(on, D, 0.0))
        Wl = np.abs(np.asarray(Ws[l - 1], dtype=np.float64))
        d_agg = np.zeros_like(D)
        for k, idx in enumerate(lg.members):
            kk = 0 if spec.weight_sharing else k
            if on_k[k]:
                sWs[l - 1][kk] += np.abs(cache["Agg"][l][idx]).T @ dG_Z[idx]
            d_agg[idx] = dG_Z[idx] @ Wl[kk].T
        D = lg.A_hat.T @ d_agg
    return D, sWs
