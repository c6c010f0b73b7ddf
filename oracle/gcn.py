"""Checker for the per-subgraph GCN training step (fp64, CPU, numpy).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
device library must compute.  It is imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, never by the product path, and it
shares no code with the HIP sources.

Everything is in ORIGINAL node order and float64.  The steps follow the paper's
Sec. 3.2 in its order and notation:

  graph convolution   h_i = sigma( (1/(|N(i)|+1)) (x_i + sum_{j in N(i)} x_j) W )   (Eq. 3)
  read-out            p_i = 1 / (1 + exp(-h_i))                                      (Eq. 4)
  loss                L = alpha * sum_{(i,j) in E} p_i p_j - beta * sum_i p_i        (Eq. 5)
  training            back-propagation, repeated for a fixed number of epochs       (Sec. 3.2, last paragraph)
  independence        every subgraph is trained on its own edges only, with its
                      own network                                                    (Sec. 3.3, first paragraph; Alg. 1 stage 1)

Readings taken where the paper is open (listed with reasons in the design notes):
  * N(i) is the neighbourhood INSIDE i's subgraph (cut edges are not trained on).
  * normalisation "mean" is Eq. 3 as printed, (D+I)^-1 (A+I); "sym" is
    (D+I)^-1/2 (A+I) (D+I)^-1/2, the form the workloads prescribe.
  * sigma = ReLU on hidden layers; the last layer is linear and scalar and feeds
    the sigmoid of Eq. 4 (ReLU before the sigmoid would pin every p_i >= 0.5).
  * L layers, L in {1,2,3}: L-1 hidden layers of Eq. 3 followed by the scalar one.
  * each undirected edge is counted once in Eq. 5.
  * the generic QUBO of Alg. 1 is L = sum_i p_i (c_i + (q/2) s_i), s = A_loc p:
    MIS has c_i = -beta, q = alpha; Max-Cut has c_i = -deg_i, q = 2, which is
    sum_{(i,j) in E_loc} (2 p_i p_j - p_i - p_j).
  * embeddings and all weight matrices are trained with Adam (beta1 0.9,
    beta2 0.999, eps 1e-8, no weight decay), one network per subgraph unless
    weights are declared shared.

Reduced-precision storage.  Three of the workloads prescribe "bf16 features with
fp32 accumulate" (one of them "X.W on bf16 MFMA").  With Spec.storage = "bf16" the
checker keeps its fp64 arithmetic but rounds to bfloat16 (8 significant bits, round
to nearest even) the tensors that such a run holds in bf16: the working copy of the
embeddings, every hidden activation H_l, the activation gradient kept between two
hidden layers, and the two operands of each hidden layer's dense transform (a bf16
matrix multiply takes bf16 operands by definition; accumulation stays unrounded).
This matters because ReLU turns a floating-point value into a yes/no decision, and a
decision has to be taken on values of the same precision on both sides of a
comparison.  Spec.storage = "exact" (default) rounds nothing.

A library routine is used for two steps only: dense matmul (numpy @) and sparse
matrix times dense matrix (scipy.sparse CSR @).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import scipy.sparse as sp


@dataclass
class Spec:
    problem: str = "mis"          # "mis" | "maxcut"
    num_layers: int = 2           # L
    norm: str = "sym"             # "sym" | "mean"
    alpha: float = 2.0
    beta: float = 1.0
    weight_sharing: bool = False  # False: one W_l per subgraph (the paper's reading)
    train_embed: bool = True
    lr: float = 1e-2
    adam_b1: float = 0.9
    adam_b2: float = 0.999
    adam_eps: float = 1e-8
    storage: str = "exact"        # "exact" | "bf16" (see the module docstring)


def round_bf16(x):
    """Round fp64 values to the nearest bfloat16 (ties to even), returned as fp64.

    bfloat16 is the upper half of an IEEE binary32: 1 sign, 8 exponent and 7
    fraction bits.  The value is first rounded to binary32 (as the device holds
    it before storing), then its low 16 bits are rounded away."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        bits = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return bits.view(np.float32).astype(np.float64).reshape(np.shape(x))


def _stored(x, spec):
    return round_bf16(x) if spec.storage == "bf16" else x


def _operand(x, spec):
    """An operand of a hidden layer's dense transform."""
    return round_bf16(x) if spec.storage == "bf16" else x


def gumbel_softmax_rows(E, U, tau):
    """Sec. 3.2: the initial embeddings are passed once through the Gumbel-softmax, which
    turns every row into a distribution close to a one-hot vector.  With noise
    g = -log(-log(u)) from given uniforms u in (0, 1) and temperature tau,
        x[i, :] = softmax((E[i, :] + g[i, :]) / tau).
    The noise is drawn once (it is an input here) and stays fixed during training."""
    E = np.asarray(E, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    g = -np.log(-np.log(U))
    y = (E + g) / float(tau)
    y = y - y.max(axis=1, keepdims=True)
    w = np.exp(y)
    return w / w.sum(axis=1, keepdims=True)


@dataclass
class LocalGraph:
    """What the training step sees of (graph, partition ids)."""
    n: int
    num_parts: int
    part: np.ndarray                 # int [n]
    A_loc: sp.csr_matrix             # 0/1 symmetric adjacency of local edges, no diagonal
    deg: np.ndarray                  # local degree, float64 [n]
    A_hat: sp.csr_matrix             # normalised (A_loc + I)
    members: list = field(default_factory=list)  # members[k] = node ids of subgraph k, ascending


def local_graph(n, rowptr, col, part, num_parts, norm) -> LocalGraph:
    """Drop cut edges, take local degrees, and normalise (Eq. 3's 1/(|N(i)|+1))."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    part = np.zeros(n, dtype=np.int64) if part is None else np.asarray(part, dtype=np.int64)
    row = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    same = part[row] == part[col]
    A_loc = sp.csr_matrix((np.ones(int(same.sum())), (row[same], col[same])), shape=(n, n))
    deg = np.asarray(A_loc.sum(axis=1)).ravel()
    d_tilde = deg + 1.0                      # |N(i)| + 1
    A_plus_I = (A_loc + sp.identity(n, format="csr")).tocsr()
    if norm == "mean":
        A_hat = sp.diags(1.0 / d_tilde) @ A_plus_I
    elif norm == "sym":
        s = 1.0 / np.sqrt(d_tilde)
        A_hat = sp.diags(s) @ A_plus_I @ sp.diags(s)
    else:
        raise ValueError(norm)
    members = [np.flatnonzero(part == k) for k in range(num_parts)]
    return LocalGraph(n, num_parts, part, A_loc.tocsr(), deg, A_hat.tocsr(), members)


def _w(W, k, spec):
    return W[0] if spec.weight_sharing else W[k]


def _apply_weights(lg: LocalGraph, X, W, spec):
    """rows of subgraph k times W[k]."""
    out = np.zeros((lg.n, W.shape[2]))
    for k, idx in enumerate(lg.members):
        out[idx] = X[idx] @ _w(W, k, spec)
    return out


def forward(lg: LocalGraph, E, Ws, spec: Spec) -> dict:
    """Eq. 3 for the hidden layers, then the scalar layer and Eq. 4."""
    L = spec.num_layers
    H = [_stored(np.asarray(E, dtype=np.float64), spec)]
    Agg, Z = [None], [None]
    for l in range(1, L):
        agg = _operand(lg.A_hat @ H[l - 1], spec)               # aggregate
        Wl = _operand(np.asarray(Ws[l - 1], dtype=np.float64), spec)
        z = _apply_weights(lg, agg, Wl, spec)                   # transform
        Agg.append(agg)
        Z.append(z)
        H.append(_stored(np.maximum(z, 0.0), spec))             # sigma = ReLU
    agg = lg.A_hat @ H[L - 1]
    z_out = _apply_weights(lg, agg, np.asarray(Ws[L - 1], dtype=np.float64), spec)[:, 0]
    Agg.append(agg)
    p = 1.0 / (1.0 + np.exp(-z_out))                            # Eq. 4
    return {"H": H, "Agg": Agg, "Z": Z, "z": z_out, "p": p}


def qubo_coefficients(lg: LocalGraph, spec: Spec):
    if spec.problem == "mis":
        return np.full(lg.n, -spec.beta), spec.alpha
    if spec.problem == "maxcut":
        return -lg.deg.copy(), 2.0
    raise ValueError(spec.problem)


def loss(lg: LocalGraph, p, spec: Spec, extra_linear=None):
    """Eq. 5 (or its generic-QUBO form): total and per-subgraph values.

    extra_linear, if given, is added to the linear coefficients c (the
    fine-tuning penalty of Sec. 3.3 has exactly this form)."""
    c, q = qubo_coefficients(lg, spec)
    if extra_linear is not None:
        c = c + extra_linear
    s = lg.A_loc @ p
    per_node = p * (c + 0.5 * q * s)
    per_part = np.array([per_node[idx].sum() for idx in lg.members])
    return float(per_part.sum()), per_part


def backward(lg: LocalGraph, cache: dict, Ws, spec: Spec, extra_linear=None, active=None,
             trace: dict = None):
    """Exact chain rule through Eq. 5, Eq. 4 and the layers of Eq. 3.

    Returns (gE [n, d], [gW_1 .. gW_L]) with gW_l shaped like W_l.

    active, if given, is a boolean array over the subgraphs: only the listed subgraphs
    contribute to the weight gradients (this matters only when the weights are shared;
    with per-subgraph weights a subgraph's gradient never depends on the others).

    trace, if given, receives "G_H": the list, indexed by hidden layer l, of dL/dH_l (the
    gradient that arrives at the ReLU of layer l)."""
    on_k = np.ones(lg.num_parts, dtype=bool) if active is None else np.asarray(active, dtype=bool)
    L = spec.num_layers
    c, q = qubo_coefficients(lg, spec)
    if extra_linear is not None:
        c = c + extra_linear
    p = cache["p"]
    s = lg.A_loc @ p
    g_p = c + q * s                                   # dL/dp_i
    g_z = g_p * p * (1.0 - p)                         # through the sigmoid
    gWs = [np.zeros_like(np.asarray(W, dtype=np.float64)) for W in Ws]
    # scalar layer: z = (A_hat H_{L-1}) w_L
    WL = np.asarray(Ws[L - 1], dtype=np.float64)
    g_agg = np.zeros_like(cache["Agg"][L])
    for k, idx in enumerate(lg.members):
        kk = 0 if spec.weight_sharing else k
        if on_k[k]:
            gWs[L - 1][kk, :, 0] += cache["Agg"][L][idx].T @ g_z[idx]
        g_agg[idx] = np.outer(g_z[idx], WL[kk, :, 0])
    g_H = lg.A_hat.T @ g_agg
    G_H = [None] * L
    for l in range(L - 1, 0, -1):
        G_H[l] = g_H
        g_Z = g_H * (cache["Z"][l] > 0.0)             # ReLU, derivative 0 at 0
        if l < L - 1:
            g_Z = _stored(g_Z, spec)                  # kept in memory between two layers
        Wl = np.asarray(Ws[l - 1], dtype=np.float64)
        g_agg = np.zeros_like(cache["Agg"][l])
        for k, idx in enumerate(lg.members):
            kk = 0 if spec.weight_sharing else k
            if on_k[k]:
                gWs[l - 1][kk] += cache["Agg"][l][idx].T @ g_Z[idx]
            g_agg[idx] = g_Z[idx] @ Wl[kk].T
        g_H = lg.A_hat.T @ g_agg
    if trace is not None:
        trace["G_H"] = G_H
    return g_H, gWs


def adam_update(theta, g, m, v, t, spec: Spec):
    """One Adam step (Kingma and Ba 2015, Alg. 1), t counted from 1."""
    m = spec.adam_b1 * m + (1.0 - spec.adam_b1) * g
    v = spec.adam_b2 * v + (1.0 - spec.adam_b2) * g * g
    m_hat = m / (1.0 - spec.adam_b1 ** t)
    v_hat = v / (1.0 - spec.adam_b2 ** t)
    theta = theta - spec.lr * m_hat / (np.sqrt(v_hat) + spec.adam_eps)
    return theta, m, v


@dataclass
class TrainState:
    """Parameters, Adam moments and Adam step counts.  Every subgraph is a model of its
    own (Alg. 1 trains and stores them one by one), so the embedding rows of subgraph k
    count their steps in tE[k] and weight set kw in tW[kw]."""
    E: np.ndarray
    Ws: list
    mE: np.ndarray
    vE: np.ndarray
    mW: list
    vW: list
    tE: np.ndarray = None
    tW: np.ndarray = None


def init_state(E, Ws) -> TrainState:
    E = np.array(E, dtype=np.float64)
    Ws = [np.array(W, dtype=np.float64) for W in Ws]
    return TrainState(E, Ws, np.zeros_like(E), np.zeros_like(E),
                      [np.zeros_like(W) for W in Ws], [np.zeros_like(W) for W in Ws])


class BestState:
    """Parameters of the lowest loss seen so far, per model (Alg. 1 stage 1: each worker
    stores the best network of its subgraph).  A model is one subgraph with its own
    weights, or, with shared weights, the whole batch judged by the total loss.  A
    subgraph without nodes has no model."""

    def __init__(self, lg: LocalGraph, st: "TrainState"):
        self.num_models = st.Ws[0].shape[0]
        self.loss = np.full(self.num_models, np.inf)
        self.E = np.zeros_like(st.E)
        self.Ws = [np.zeros_like(W) for W in st.Ws]

    def offer(self, lg: LocalGraph, st: "TrainState", per_part, on_k):
        """Called with the losses of the parameters `st` holds right now."""
        if self.num_models == lg.num_parts:
            for k, idx in enumerate(lg.members):
                if on_k[k] and len(idx) and per_part[k] < self.loss[k]:
                    self.loss[k] = per_part[k]
                    self.E[idx] = st.E[idx]
                    for l, W in enumerate(st.Ws):
                        self.Ws[l][k] = W[k]
        else:
            total = per_part[on_k].sum()
            if on_k.any() and total < self.loss[0]:
                self.loss[0] = total
                self.E[...] = st.E
                for l, W in enumerate(st.Ws):
                    self.Ws[l][...] = W

    def restore(self, lg: LocalGraph, st: "TrainState"):
        """Put the stored parameters back (models without a snapshot keep theirs)."""
        if self.num_models == lg.num_parts:
            for k, idx in enumerate(lg.members):
                if np.isfinite(self.loss[k]):
                    st.E[idx] = self.E[idx]
                    for l in range(len(st.Ws)):
                        st.Ws[l][k] = self.Ws[l][k]
        elif np.isfinite(self.loss[0]):
            st.E[...] = self.E
            for l in range(len(st.Ws)):
                st.Ws[l][...] = self.Ws[l]


def train(lg: LocalGraph, st: TrainState, spec: Spec, epochs: int, extra_linear=None, active=None,
          best: BestState = None):
    """`epochs` full-batch steps of the subgraphs listed in `active` (boolean array over the
    subgraphs; None = all): Sec. 3.2 for all of them, the fine-tuning step of Sec. 3.3 /
    Alg. 1 stage 3 for a subset.  Subgraphs that are not listed keep parameters, moments
    and step counts.  Returns the loss (summed over the listed subgraphs) at the parameters
    each epoch started from, and per-subgraph losses [epochs, P].  With `best`, every
    epoch's losses are offered to it together with the parameters they belong to (those
    the epoch started from)."""
    P, Pw = lg.num_parts, st.Ws[0].shape[0]
    if st.tE is None:
        st.tE = np.zeros(P, dtype=np.int64)
        st.tW = np.zeros(Pw, dtype=np.int64)
    on_k = np.ones(P, dtype=bool) if active is None else np.asarray(active, dtype=bool)
    on_w = on_k if Pw == P else np.array([on_k.any()])
    losses, per_part = [], []
    for _ in range(epochs):
        cache = forward(lg, st.E, st.Ws, spec)
        _, pp = loss(lg, cache["p"], spec, extra_linear)
        losses.append(pp[on_k].sum())
        per_part.append(pp)
        if best is not None:
            best.offer(lg, st, pp, on_k)
        gE, gWs = backward(lg, cache, st.Ws, spec, extra_linear, active=on_k)
        st.tE[on_k] += 1
        st.tW[on_w] += 1
        if spec.train_embed:
            for k, idx in enumerate(lg.members):
                if on_k[k]:
                    st.E[idx], st.mE[idx], st.vE[idx] = adam_update(
                        st.E[idx], gE[idx], st.mE[idx], st.vE[idx], int(st.tE[k]), spec)
        for l in range(spec.num_layers):
            for kw in range(Pw):
                if on_w[kw]:
                    st.Ws[l][kw], st.mW[l][kw], st.vW[l][kw] = adam_update(
                        st.Ws[l][kw], gWs[l][kw], st.mW[l][kw], st.vW[l][kw], int(st.tW[kw]), spec)
    return np.array(losses), np.array(per_part)
