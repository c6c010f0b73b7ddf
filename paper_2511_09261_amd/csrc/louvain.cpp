// Graph partitioning by modularity (Sec. 3.1): the Louvain heuristic on the host.
//
// Gains are compared as the integers 2 m^2 dQ = 2 m k_ic - tot_c k_i (Sec. 3.1, Eq. 2), so
// the result does not depend on floating-point rounding.  Deterministic rules: nodes are
// visited in ascending id, sweep after sweep, until a sweep moves nothing; a node leaves its
// community for the neighbouring community of largest gain only if that gain is strictly
// larger than the gain of going back; ties go to the smallest community id; communities
// become the nodes of the next level, numbered by their smallest member; the levels end
// when a level moves nothing.  Final ids are numbered by smallest original member.
#include <algorithm>
#include <cstdint>
#include <functional>
#include <queue>
#include <utility>
#include <vector>

#include "gco.h"

namespace {

struct Level {
  std::vector<int64_t> ptr;   // [N+1]
  std::vector<int32_t> nbr;   // neighbours j != i
  std::vector<int64_t> w;     // edge weights
  std::vector<int64_t> self;  // weight of the edges inside a super-node, each once
  int32_t size() const { return static_cast<int32_t>(self.size()); }
};

// One level of local moving; comm[i] = community of node i.  Returns whether anything moved.
bool local_moving(const Level& g, int64_t m, std::vector<int32_t>& comm) {
  const int32_t N = g.size();
  std::vector<int64_t> k(N), tot(N), w_to(N, 0);
  std::vector<int32_t> touched;
  for (int32_t i = 0; i < N; ++i) {
    int64_t d = 2 * g.self[i];
    for (int64_t e = g.ptr[i]; e < g.ptr[i + 1]; ++e) d += g.w[e];
    k[i] = d;
    tot[i] = d;
    comm[i] = i;
  }
  bool moved_any = false;
  while (true) {
    bool moved = false;
    for (int32_t i = 0; i < N; ++i) {
      const int32_t old = comm[i];
      touched.clear();
      for (int64_t e = g.ptr[i]; e < g.ptr[i + 1]; ++e) {
        const int32_t c = comm[g.nbr[e]];
        if (w_to[c] == 0) touched.push_back(c);
        w_to[c] += g.w[e];
      }
      tot[old] -= k[i];
      // 2 m^2 dQ of joining community c (Eq. 2); fits 64 bits: both products are <= (2m)^2
      auto gain = [&](int32_t c) { return 2 * m * w_to[c] - tot[c] * k[i]; };
      int32_t best_c = old;
      int64_t best_g = gain(old);
      for (int32_t c : touched) {
        const int64_t gc = gain(c);
        if (gc > best_g || (gc == best_g && best_c != old && c < best_c)) {
          best_c = c;
          best_g = gc;
        }
      }
      for (int32_t c : touched) w_to[c] = 0;
      comm[i] = best_c;
      tot[best_c] += k[i];
      if (best_c != old) moved = true;
    }
    if (!moved) break;
    moved_any = true;
  }
  return moved_any;
}

// Communities -> nodes of the next level, numbered by smallest member; new_of[i] = new node.
Level aggregate(const Level& g, const std::vector<int32_t>& comm, std::vector<int32_t>& new_of) {
  const int32_t N = g.size();
  std::vector<int32_t> id(N, -1);
  int32_t N2 = 0;
  new_of.resize(N);
  for (int32_t i = 0; i < N; ++i) {
    if (id[comm[i]] < 0) id[comm[i]] = N2++;
    new_of[i] = id[comm[i]];
  }
  // members of every new node, in ascending old id
  std::vector<int64_t> mptr(static_cast<size_t>(N2) + 1, 0);
  for (int32_t i = 0; i < N; ++i) mptr[new_of[i] + 1]++;
  for (int32_t a = 0; a < N2; ++a) mptr[a + 1] += mptr[a];
  std::vector<int32_t> members(N);
  {
    std::vector<int64_t> cur(mptr.begin(), mptr.end() - 1);
    for (int32_t i = 0; i < N; ++i) members[cur[new_of[i]]++] = i;
  }
  Level out;
  out.self.assign(N2, 0);
  out.ptr.assign(static_cast<size_t>(N2) + 1, 0);
  std::vector<int64_t> acc(N2, 0);
  std::vector<int32_t> touched;
  for (int32_t a = 0; a < N2; ++a) {
    touched.clear();
    for (int64_t q = mptr[a]; q < mptr[a + 1]; ++q) {
      const int32_t i = members[q];
      out.self[a] += g.self[i];
      for (int64_t e = g.ptr[i]; e < g.ptr[i + 1]; ++e) {
        const int32_t j = g.nbr[e], b = new_of[j];
        if (b == a) {
          if (i < j) out.self[a] += g.w[e];
        } else {
          if (acc[b] == 0) touched.push_back(b);
          acc[b] += g.w[e];
        }
      }
    }
    std::sort(touched.begin(), touched.end());
    for (int32_t b : touched) {
      out.nbr.push_back(b);
      out.w.push_back(acc[b]);
      acc[b] = 0;
    }
    out.ptr[a + 1] = static_cast<int64_t>(out.nbr.size());
  }
  return out;
}

}  // namespace

extern "C" int gco_louvain(int64_t n64, const int64_t* rowptr, const int32_t* col, int32_t max_levels,
                           int32_t* part_id, int32_t* num_parts, double* modularity) {
  if (n64 < 1 || n64 >= (int64_t{1} << 31) || !rowptr || !part_id || max_levels < 0) return GCO_EINVAL;
  const int32_t n = static_cast<int32_t>(n64);
  if (rowptr[0] != 0) return GCO_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (rowptr[i + 1] < rowptr[i]) return GCO_EINVAL;
  const int64_t nnz = rowptr[n];
  if (nnz > 0 && !col) return GCO_EINVAL;
  if (nnz % 2 != 0 || nnz >= (int64_t{1} << 31)) return nnz % 2 ? GCO_EINVAL : GCO_ERANGE;
  for (int64_t e = 0; e < nnz; ++e)
    if (col[e] < 0 || col[e] >= n) return GCO_EINVAL;
  const int64_t m = nnz / 2;

  Level g;
  g.ptr.assign(rowptr, rowptr + n + 1);
  g.nbr.assign(col, col + nnz);
  g.w.assign(static_cast<size_t>(nnz), 1);
  g.self.assign(n, 0);
  for (int32_t i = 0; i < n; ++i)
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
      if (col[e] == i) return GCO_EINVAL;  // self loop
  std::vector<int32_t> member_of(n);
  for (int32_t i = 0; i < n; ++i) member_of[i] = i;
  if (m > 0) {
    std::vector<int32_t> comm, new_of;
    for (int32_t level = 0; level < max_levels; ++level) {
      comm.assign(g.size(), 0);
      if (!local_moving(g, m, comm)) break;
      Level next = aggregate(g, comm, new_of);
      for (int32_t i = 0; i < n; ++i) member_of[i] = new_of[member_of[i]];
      g = std::move(next);
    }
  }
  // ids by smallest original member
  std::vector<int32_t> final_id(g.size(), -1);
  int32_t P = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (final_id[member_of[i]] < 0) final_id[member_of[i]] = P++;
    part_id[i] = final_id[member_of[i]];
  }
  if (num_parts) *num_parts = P;
  if (modularity) {
    // Q = sum_c in_c / m - (tot_c / 2m)^2 from the last level's nodes (fp64)
    double q = 0.0;
    if (m > 0) {
      std::vector<double> in_c(P, 0.0), tot_c(P, 0.0);
      for (int32_t i = 0; i < n; ++i) {
        const int32_t c = part_id[i];
        tot_c[c] += static_cast<double>(rowptr[i + 1] - rowptr[i]);
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
          if (part_id[col[e]] == c && col[e] > i) in_c[c] += 1.0;
      }
      for (int32_t c = 0; c < P; ++c)
        q += in_c[c] / static_cast<double>(m) - (tot_c[c] / (2.0 * m)) * (tot_c[c] / (2.0 * m));
    }
    *modularity = q;
  }
  return GCO_OK;
}

extern "C" int gco_pack_parts(int64_t n, const int32_t* part_id, int32_t num_parts, int32_t max_parts,
                              int32_t* part_out, int32_t* num_out) {
  if (n < 0 || !part_id || !part_out || num_parts < 1 || max_parts < 1) return GCO_EINVAL;
  for (int64_t i = 0; i < n; ++i)
    if (part_id[i] < 0 || part_id[i] >= num_parts) return GCO_EINVAL;
  if (num_parts <= max_parts) {
    for (int64_t i = 0; i < n; ++i) part_out[i] = part_id[i];
    if (num_out) *num_out = num_parts;
    return GCO_OK;
  }
  std::vector<int64_t> size(num_parts, 0);
  for (int64_t i = 0; i < n; ++i) size[part_id[i]]++;
  std::vector<int32_t> order(num_parts);
  for (int32_t c = 0; c < num_parts; ++c) order[c] = c;
  std::sort(order.begin(), order.end(),
            [&](int32_t a, int32_t b) { return size[a] != size[b] ? size[a] > size[b] : a < b; });
  // the group with the smallest (load, id) is on top
  typedef std::pair<int64_t, int32_t> Bin;
  std::priority_queue<Bin, std::vector<Bin>, std::greater<Bin>> bins;
  for (int32_t b = 0; b < max_parts; ++b) bins.push(Bin(0, b));
  std::vector<int32_t> group(num_parts);
  for (int32_t c : order) {
    Bin top = bins.top();
    bins.pop();
    group[c] = top.second;
    top.first += size[c];
    bins.push(top);
  }
  for (int64_t i = 0; i < n; ++i) part_out[i] = group[part_id[i]];
  if (num_out) *num_out = max_parts;
  return GCO_OK;
}
