"""Checker for the cross-subgraph coordination stage (fp64, CPU).

TEST INFRASTRUCTURE ONLY (see oracle/gcn.py): imported by tests, never by the product
path, no code shared with the library.

Sec. 3.3 and Alg. 1 stage 3 of the paper, for Maximum Independent Set: after every
subgraph has been trained on its own, the cross edges (ends in different subgraphs) whose
two ends are both selected are CONFLICTS.  For a conflict (i, j) there are two options:
fine-tune i's subgraph so that p_i falls below 0.5, or j's so that p_j does.  Fine-tuning
adds lambda * (sum of the selected nodes' probabilities) to the subgraph's loss.  A
Q-learning agent picks which options to apply over T rounds; the best assignment seen is
kept.

The paper leaves most of the stage open.  PARITY UNPINNED: no printed value, closed form or
invariant fixes the choices below; they are one reading of the paper, written down once here
and followed step by step by the library's gco_coordinate, so the two can be compared
decision by decision.

  score        the negated objective of the whole graph on the binarised assignment:
               score(x) = beta |S| - alpha #{edges of the WHOLE graph inside S}  (Eq. 5 at p = x)
  base action  (Alg. 1 stage 3 starts the agent from a linear-time cover): one pass over the
               current conflict edges in (u, v) order; an edge with an end already chosen
               is covered; otherwise the end with the smaller probability (compared in
               fp32; ties: smaller id) is chosen.  The chosen nodes cover every conflict.
  diff         (the difference to the base action that the agent selects): either nothing, or the other end at ONE of the edges where
               the pass made a choice; the pass is then redone with that choice forced.
  state        the assignment restricted to the ends of the FIRST round's conflict edges
               (Sec. 3.3: binarised cross-node probabilities).
  agent        tabular Q over (state, diff), diff named by the node it brings in (-1: none);
               epsilon-greedy from uniforms the caller supplies (two per round); greedy
               ties go to the earlier candidate; unseen entries are 0;
               Q(s, a) += eta (r + gamma max_a' Q(s', a') - Q(s, a)), r = score' - score.
  fine-tune    the chosen nodes get the penalty lambda for good (penalties accumulate);
               the subgraphs that own this round's chosen nodes train `epochs` epochs.
  best         the assignment of the highest score, the first one on ties.
The stage stops early when no conflict is left.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import combinatorial as cb
from . import gcn


@dataclass
class RLSpec:
    rounds: int = 10
    epochs: int = 5          # fine-tuning epochs per round
    lam: float = 1.0         # penalty coefficient lambda of Sec. 3.3
    q_lr: float = 0.5        # eta
    q_gamma: float = 0.9
    epsilon: float = 0.2


def score(n, rowptr, col, x, alpha, beta):
    inside = cb.count_conflicts(n, rowptr, col, None, x, "all")
    return beta * float(x.sum()) - alpha * float(inside)


def linear_cover(cu, cv, p32, forced=-1):
    """The pass described above.  forced = index of a conflict edge at which the OTHER end
    is taken if the pass has to choose there.  Returns (chosen nodes in the order chosen,
    indices of the edges at which a choice was made, the end NOT chosen at each of them)."""
    chosen, chosen_set, at, other = [], set(), [], []
    for e in range(len(cu)):
        u, v = int(cu[e]), int(cv[e])
        if u in chosen_set or v in chosen_set:
            continue
        pick = u if (p32[u] < p32[v] or (p32[u] == p32[v] and u < v)) else v
        if e == forced:
            pick = v if pick == u else u
        chosen.append(pick)
        chosen_set.add(pick)
        at.append(e)
        other.append(v if pick == u else u)
    return chosen, at, other


def coordinate(n, rowptr, col, part, lg: gcn.LocalGraph, st: gcn.TrainState, spec: gcn.Spec,
               rl: RLSpec, uniforms):
    """Runs the stage on the checker's own training state `st` (trained in place).
    uniforms: array [rounds, 2] of numbers in [0, 1).  Returns a dict with x_best,
    score_best, scores (one per evaluated assignment), actions (node brought in by the
    diff of every round run, -1 for none), chosen (the penalised nodes of every round),
    conflicts (cross conflicts of every evaluated assignment)."""
    assert spec.problem == "mis"
    uniforms = np.asarray(uniforms, dtype=np.float64).reshape(-1, 2)
    cut_u, cut_v = cb.cut_edges_vectorised(n, rowptr, col, part)
    part = np.asarray(part)
    pen = np.zeros(n, dtype=np.float64)

    def evaluate():
        p32 = gcn.forward(lg, st.E, st.Ws, spec)["p"].astype(np.float32)
        x = cb.round_probs(p32)
        cu, cv = cb.conflict_edges(cut_u, cut_v, x)
        return p32, x, cu, cv, score(n, rowptr, col, x, spec.alpha, spec.beta)

    p32, x, cu, cv, sc = evaluate()
    ends = np.unique(np.concatenate([cu, cv])).astype(np.int64)     # state: these nodes' bits
    state = x[ends].tobytes()
    Q = {}
    out = {"scores": [sc], "conflicts": [len(cu)], "actions": [], "chosen": [],
           "x_best": x.copy(), "score_best": sc}
    for t in range(rl.rounds):
        if len(cu) == 0:
            break
        _, at, other = linear_cover(cu, cv, p32)
        candidates = [(-1, -1)] + [(other[q], at[q]) for q in range(len(at))]   # (node brought in, forced edge)
        if uniforms[t, 0] < rl.epsilon:
            pick = min(int(uniforms[t, 1] * len(candidates)), len(candidates) - 1)
        else:
            values = [Q.get((state, a), 0.0) for a, _ in candidates]
            pick = int(np.argmax(values))                                       # first maximum
        action, forced = candidates[pick]
        chosen, _, _ = linear_cover(cu, cv, p32, forced)
        pen[chosen] = rl.lam
        active = np.zeros(lg.num_parts, dtype=bool)
        active[part[chosen]] = True
        gcn.train(lg, st, spec, rl.epochs, extra_linear=pen, active=active)
        p32, x, cu, cv, sc_new = evaluate()
        new_state = x[ends].tobytes()
        reward = sc_new - sc
        future = max([0.0] + [v for (s, _), v in Q.items() if s == new_state])
        old = Q.get((state, action), 0.0)
        Q[(state, action)] = old + rl.q_lr * (reward + rl.q_gamma * future - old)
        state, sc = new_state, sc_new
        out["scores"].append(sc)
        out["conflicts"].append(len(cu))
        out["actions"].append(action)
        out["chosen"].append(sorted(chosen))
        if sc > out["score_best"]:
            out["score_best"] = sc
            out["x_best"] = x.copy()
    out["Q"] = Q
    return out
