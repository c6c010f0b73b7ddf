// Cross-subgraph coordination (Sec. 3.3; Alg. 1 stage 3) as a thin host-side consumer of the
// C ABI: everything below goes through the public calls of include/gco.h (forward,
// probabilities, binarisation with the conflict count, cross edges, per-node penalty,
// training of a subset of the subgraphs).  No kernel of its own.
//
// What the paper leaves open (state, reward, schedule, the "linear cover") is fixed as
// described at gco_coordinate in include/gco.h.
#include <algorithm>
#include <cstdint>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "gco.h"

namespace {

struct Cover {
  std::vector<int32_t> chosen;  // nodes that receive the penalty, in the order chosen
  std::vector<int32_t> at;      // conflict edges at which the pass had to choose
  std::vector<int32_t> other;   // the end it did not take there
};

// One pass over the conflict edges (u[e], v[e]) in list order: an edge with an end already
// chosen is covered; otherwise the end with the smaller probability is chosen (ties: the
// smaller id); at edge `forced` the other end is taken instead.
Cover linear_cover(const std::vector<int32_t>& u, const std::vector<int32_t>& v, const std::vector<float>& p,
                   std::vector<uint8_t>& mark, int64_t forced) {
  Cover c;
  for (size_t e = 0; e < u.size(); ++e) {
    const int32_t a = u[e], b = v[e];
    if (mark[a] || mark[b]) continue;
    int32_t pick = (p[a] < p[b] || (p[a] == p[b] && a < b)) ? a : b;
    if (static_cast<int64_t>(e) == forced) pick = pick == a ? b : a;
    mark[pick] = 1;
    c.chosen.push_back(pick);
    c.at.push_back(static_cast<int32_t>(e));
    c.other.push_back(pick == a ? b : a);
  }
  for (int32_t i : c.chosen) mark[i] = 0;
  return c;
}

}  // namespace

extern "C" int gco_coordinate(gco_ctx* ctx, const int32_t* part_id, const gco_rl_config* rl,
                              const double* uniforms, uint8_t* x_best, double* score_best,
                              int32_t* actions, double* scores, int64_t* conflicts, int32_t* rounds_run) {
  if (!ctx || !rl || !x_best) return GCO_EINVAL;
  if (rl->rounds < 0 || rl->epochs_per_round < 0 || !(rl->lambda >= 0.f)) return GCO_EINVAL;
  if (rl->rounds > 0 && !uniforms) return GCO_EINVAL;
  gco_config cfg;
  int rc = gco_get_config(ctx, &cfg);
  if (rc != GCO_OK) return rc;
  if (cfg.problem != GCO_PROBLEM_MIS) return GCO_EINVAL;  // conflicts are defined for independent sets
  int64_t n64 = 0;
  rc = gco_graph_info(ctx, &n64, nullptr, nullptr, nullptr);
  if (rc != GCO_OK) return rc;
  const size_t n = static_cast<size_t>(n64);

  // cross edges, once
  int64_t num_cut = 0;
  rc = gco_cut_edges(ctx, &num_cut, nullptr, nullptr);
  if (rc != GCO_OK) return rc;
  std::vector<int32_t> cut_u(static_cast<size_t>(num_cut)), cut_v(static_cast<size_t>(num_cut));
  if (num_cut > 0) {
    rc = gco_cut_edges(ctx, &num_cut, cut_u.data(), cut_v.data());
    if (rc != GCO_OK) return rc;
  }

  std::vector<float> p(n), pen(n, 0.f);
  std::vector<uint8_t> x(n), mark(n, 0);
  std::vector<int32_t> cu, cv;
  const float alpha = cfg.alpha, beta = cfg.beta;

  // forward, binarise, conflicts among the cross edges, score of the whole graph
  auto evaluate = [&](double* sc) -> int {
    int r = gco_forward(ctx);
    if (r != GCO_OK) return r;
    if ((r = gco_get_probs(ctx, p.data())) != GCO_OK) return r;
    int64_t size = 0, inside = 0;
    if ((r = gco_round_repair(ctx, 0.5f, GCO_REPAIR_NONE, x.data(), &size, &inside, nullptr)) != GCO_OK) return r;
    cu.clear();
    cv.clear();
    for (size_t e = 0; e < cut_u.size(); ++e)
      if (x[cut_u[e]] && x[cut_v[e]]) {
        cu.push_back(cut_u[e]);
        cv.push_back(cut_v[e]);
      }
    *sc = static_cast<double>(beta) * static_cast<double>(size) - static_cast<double>(alpha) * static_cast<double>(inside);
    return GCO_OK;
  };

  double sc = 0.0;
  if ((rc = evaluate(&sc)) != GCO_OK) return rc;
  // the agent's state: the assignment on the ends of the first round's conflicts
  std::vector<int32_t> ends(cu);
  ends.insert(ends.end(), cv.begin(), cv.end());
  std::sort(ends.begin(), ends.end());
  ends.erase(std::unique(ends.begin(), ends.end()), ends.end());
  auto state_of = [&]() {
    std::string s(ends.size(), '0');
    for (size_t q = 0; q < ends.size(); ++q) s[q] = x[ends[q]] ? '1' : '0';
    return s;
  };
  std::string state = state_of();
  std::map<std::pair<std::string, int32_t>, double> Q;
  auto q_of = [&](const std::string& s, int32_t a) {
    const auto it = Q.find(std::make_pair(s, a));
    return it == Q.end() ? 0.0 : it->second;
  };

  double best = sc;
  std::copy(x.begin(), x.end(), x_best);
  if (scores) scores[0] = sc;
  if (conflicts) conflicts[0] = static_cast<int64_t>(cu.size());
  int32_t t = 0;
  for (; t < rl->rounds; ++t) {
    if (cu.empty()) break;
    const Cover base = linear_cover(cu, cv, p, mark, -1);
    // candidates: no diff (node -1), or the other end at one of the choosing edges
    const size_t num_cand = base.at.size() + 1;
    size_t pick = 0;
    if (uniforms[2 * t] < static_cast<double>(rl->epsilon)) {
      pick = std::min(static_cast<size_t>(uniforms[2 * t + 1] * static_cast<double>(num_cand)), num_cand - 1);
    } else {
      double top = q_of(state, -1);
      for (size_t q = 0; q < base.at.size(); ++q) {
        const double val = q_of(state, base.other[q]);
        if (val > top) {  // the first maximum wins
          top = val;
          pick = q + 1;
        }
      }
    }
    const int32_t action = pick == 0 ? -1 : base.other[pick - 1];
    const Cover cover = pick == 0 ? base : linear_cover(cu, cv, p, mark, base.at[pick - 1]);
    // penalties accumulate; the subgraphs that own this round's nodes are fine-tuned
    std::vector<int32_t> parts;
    for (int32_t i : cover.chosen) {
      pen[i] = rl->lambda;
      parts.push_back(part_id ? part_id[i] : 0);
    }
    std::sort(parts.begin(), parts.end());
    parts.erase(std::unique(parts.begin(), parts.end()), parts.end());
    if ((rc = gco_set_linear_penalty(ctx, pen.data())) != GCO_OK) return rc;
    if ((rc = gco_train_subset(ctx, rl->epochs_per_round, parts.data(), static_cast<int32_t>(parts.size()),
                               nullptr)) != GCO_OK)
      return rc;
    double sc_new = 0.0;
    if ((rc = evaluate(&sc_new)) != GCO_OK) return rc;
    const std::string new_state = state_of();
    double future = 0.0;  // entries never written count 0
    for (const auto& kv : Q)
      if (kv.first.first == new_state) future = std::max(future, kv.second);
    const double old = q_of(state, action);
    Q[std::make_pair(state, action)] =
        old + static_cast<double>(rl->q_lr) * ((sc_new - sc) + static_cast<double>(rl->q_gamma) * future - old);
    state = new_state;
    sc = sc_new;
    if (actions) actions[t] = action;
    if (scores) scores[t + 1] = sc;
    if (conflicts) conflicts[t + 1] = static_cast<int64_t>(cu.size());
    if (sc > best) {
      best = sc;
      std::copy(x.begin(), x.end(), x_best);
    }
  }
  if (score_best) *score_best = best;
  if (rounds_run) *rounds_run = t;
  return GCO_OK;
}
